// Host runtime behind the C ABI: partition store (pinned host tier + HBM buffer slots),
// swap scheduling on a side stream, the per-bucket batch loop, reads and diagnostics.
// Paper: Sec. 3 (storage arrangement, steps 1-8), Sec. 4 (buffer of three, prefetching).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <exception>
#include <new>
#include <string>
#include <vector>

#include "legend_internal.h"
#include "device_utils.h"

using namespace legend;

static __device__ __align__(256) unsigned char scratch[(size_t)8 << 20];

namespace {

// message of the calling thread's last failure: a fixed buffer, so that reporting an error never allocates
thread_local char g_last_error[512] = "";

int fail(int code, const char* fmt, ...) noexcept {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
    va_end(ap);
    return code;
}

// Every entry point runs its body through this: no C++ exception (the containers of the host runtime
// can throw std::bad_alloc) leaves the library through the C ABI.
template <class F>
int guarded(const char* what, F&& body) noexcept {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return fail(LEGEND_E_NOMEM, "%s: out of host memory", what);
    } catch (const std::exception& e) {
        return fail(LEGEND_E_STATE, "%s: unexpected failure in the host runtime: %s", what, e.what());
    } catch (...) {
        return fail(LEGEND_E_STATE, "%s: unexpected failure in the host runtime", what);
    }
}

// Scratch memory of legend_rank_edges_static: lives in the code object, one copy per device, until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the device
// address is resolved once per device (resolve_static_scratch) and kernels and fills take that pointer.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
unsigned char* g_static_scratch[kMaxDevices] = {};

const char* kClassNames[KC_COUNT] = {"prepare", "sort", "chunk", "update", "chunk_redo", "misc", "update_long"};

struct ProfSpan {
    int cls;
    hipEvent_t a, b;
};

}  // namespace

// device address of `scratch` on the current device `dev`; resolved on first use per device
static int resolve_static_scratch(int dev) {
    if (dev < 0 || dev >= kMaxDevices) return fail(LEGEND_E_INVAL, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    if (g_static_scratch[dev]) return LEGEND_OK;
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
        (void)hipGetLastError();
        return fail(LEGEND_E_HIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
    }
    g_static_scratch[dev] = static_cast<unsigned char*>(p);
    return LEGEND_OK;
}

struct legend_ctx {
    legend_config cfg{};
    int64_t V = 0;
    int n = 0, cap = 0, d = 0;
    int64_t Rp = 0;
    size_t part_floats = 0;                 // 2 * Rp * d
    int nrel_rows = 1;
    bool uses_rel = false;
    std::vector<float*> host_part;          // pinned [E_p | S_p]
    std::vector<float*> slot_mem;           // device [E | S]
    std::vector<float*> slot_grad;          // atomic mode: device gradient accumulator per slot [Rp * d]
    float* G_rel = nullptr;
    std::vector<int> slot_part, part_slot;
    std::vector<hipEvent_t> slot_ready;
    std::vector<char> slot_pending;
    // With fewer logical slots than partitions there is one physical slot more: a partition is loaded
    // into the free slot while the evicted one is still being written back (both PCIe directions at once).
    int nslots = 0;                         // physical slots: cap, or cap + 1
    hipStream_t copy_out = nullptr;         // device-to-host write-backs
    std::vector<hipEvent_t> slot_drained;   // write-back of the slot's previous tenant complete
    std::vector<char> slot_draining;
    std::vector<int> slot_drain_part;       // the partition whose write-back slot_drained marks
    float* E_rel = nullptr;
    float* S_rel = nullptr;
    std::vector<float*> h_part_emb, h_part_state;   // host images of the two tables below (sized at init)
    float** d_part_emb = nullptr;           // device: embedding base per partition or null
    float** d_part_state = nullptr;
    hipStream_t compute = nullptr, copy = nullptr;
    bool own_compute = false, own_copy = false;
    hipEvent_t ev_fence = nullptr, ev_t0 = nullptr, ev_t1 = nullptr;
    hipStream_t aux = nullptr;              // index side (negatives, keys, sort) of the next batch, one batch ahead
    hipStream_t aux2 = nullptr;             // update of the table rows with many gradient rows, next to the other rows' update
    hipEvent_t ev_chunk_done = nullptr, ev_long_done = nullptr;
    hipEvent_t ev_start = nullptr;          // compute stream has reached the start of a bucket call
    hipEvent_t ev_index[3] = {nullptr, nullptr, nullptr};    // index side of a batch complete (per workspace)
    hipEvent_t ev_updated[3] = {nullptr, nullptr, nullptr};  // update of a batch complete: its index buffers are free
    Workspace ws{};                         // even batches of a call; also every serial path
    Workspace ws_alt[2]{};                  // batches 1 and 2 (mod 3): own index-side buffers, the rest shared with ws
    BatchGeom gmax{};
    int key_bits = 0;
    int32_t* edges_dev = nullptr;
    int64_t edges_cap = 0;
    void* io_dev = nullptr;                 // scratch for score / read calls
    size_t io_cap = 0;
    uint32_t prof_mask = 0;
    std::vector<ProfSpan> prof_spans;
    std::vector<hipEvent_t> prof_pool;
    double prof_ms[KC_COUNT] = {0};
    int64_t prof_launches[KC_COUNT] = {0};
    int64_t batches_done = 0;
    bool index_after_chunk = false;         // LEGEND_INDEX_AFTER_CHUNK=1: the next batch's index side starts when this batch's chunk kernel has finished, not when it is launched (a measurement knob)
    bool no_small_update = false;           // LEGEND_NO_SMALL_UPDATE=1: small batches take the general update kernels too (tests compare the two)
    bool serial_sort = false;               // LEGEND_SERIAL_SORT=1: everything on the compute stream, batch after batch (for per-kernel timing)
    bool keep_loss = false;                 // epoch driver: do not reset the device loss sum per bucket
    bool part_tables_dirty = false;         // d_part_emb / d_part_state lag behind part_slot
    bool fatal = false;
};

namespace {

#define HIP_TRY(ctx, expr)                                                                        \
    do {                                                                                          \
        hipError_t _e = (expr);                                                                   \
        if (_e != hipSuccess) {                                                                   \
            if (ctx) (ctx)->fatal = true;                                                         \
            return fail(LEGEND_E_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e),     \
                        __FILE__, __LINE__);                                                      \
        }                                                                                         \
    } while (0)

int64_t rows_valid(const legend_ctx* c, int part) {
    int64_t lo = (int64_t)part * c->Rp;
    return std::max<int64_t>(0, std::min<int64_t>(c->Rp, c->V - lo));
}

BatchGeom make_geom(const legend_ctx* c, int P) {
    BatchGeom g{};
    const legend_config& cf = c->cfg;
    g.P = P;
    g.C = cf.chunk_size;
    g.N = cf.num_negs;
    g.T = row_tiles_for(cf.chunk_size, c->d);
    g.rows_tile = rows_per_tile_for(cf.chunk_size, c->d);
    g.nchunks = (P + g.C - 1) / g.C;
    g.sides = cf.corrupt == LEGEND_CORRUPT_BOTH ? 2 : 1;
    g.side_id[0] = cf.corrupt == LEGEND_CORRUPT_SRC ? 1 : 0;
    g.side_id[1] = 1;
    g.roles = c->uses_rel ? 3 : 2;
    g.per_side = (int64_t)g.roles * P + (int64_t)g.nchunks * g.T * g.N;
    g.n_occ = g.per_side * g.sides;
    return g;
}

// ---- profiling ---------------------------------------------------------------------------------
hipEvent_t prof_event(legend_ctx* c) {
    if (!c->prof_pool.empty()) {
        hipEvent_t e = c->prof_pool.back();
        c->prof_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct ProfScope {
    legend_ctx* c;
    int cls;
    hipStream_t st;
    hipEvent_t a = nullptr, b = nullptr;
    ProfScope(legend_ctx* ctx, int k, hipStream_t stream = nullptr) : c(ctx), cls(k), st(stream ? stream : ctx->compute) {
        if (c->prof_mask & (1u << cls)) {
            a = prof_event(c);
            b = prof_event(c);
            if (a && b) (void)hipEventRecord(a, st);
        }
    }
    ~ProfScope() {
        if (a && b) {
            (void)hipEventRecord(b, st);
            c->prof_spans.push_back({cls, a, b});
        }
    }
};

int prof_collect(legend_ctx* c) {
    for (auto& s : c->prof_spans) {
        float ms = 0.f;
        HIP_TRY(c, hipEventSynchronize(s.b));
        HIP_TRY(c, hipEventElapsedTime(&ms, s.a, s.b));
        c->prof_ms[s.cls] += ms;
        c->prof_launches[s.cls] += 1;
        c->prof_pool.push_back(s.a);
        c->prof_pool.push_back(s.b);
    }
    c->prof_spans.clear();
    return LEGEND_OK;
}

int ensure_io(legend_ctx* c, size_t bytes) {
    if (bytes <= c->io_cap) return LEGEND_OK;
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    if (c->io_dev) HIP_TRY(c, hipFree(c->io_dev));
    c->io_dev = nullptr;
    c->io_cap = 0;
    size_t want = std::max<size_t>(bytes, 1 << 20);
    if (hipMalloc(&c->io_dev, want) != hipSuccess) return fail(LEGEND_E_NOMEM, "device scratch of %zu bytes", want);
    c->io_cap = want;
    return LEGEND_OK;
}

int upload_part_tables(legend_ctx* c) {
    std::vector<float*>& e = c->h_part_emb;
    std::vector<float*>& s = c->h_part_state;
    for (int p = 0; p < c->n; ++p) {
        int sl = c->part_slot[p];
        e[p] = sl >= 0 ? c->slot_mem[sl] : nullptr;
        s[p] = sl >= 0 ? c->slot_mem[sl] + c->Rp * c->d : nullptr;
    }
    HIP_TRY(c, hipMemcpyAsync(c->d_part_emb, e.data(), sizeof(float*) * c->n, hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, hipMemcpyAsync(c->d_part_state, s.data(), sizeof(float*) * c->n, hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    c->part_tables_dirty = false;
    return LEGEND_OK;
}

int wait_slot(legend_ctx* c, int slot) {
    if (c->slot_pending[slot]) {
        HIP_TRY(c, hipStreamWaitEvent(c->compute, c->slot_ready[slot], 0));
        c->slot_pending[slot] = 0;
    }
    return LEGEND_OK;
}

// `early_load`: the epoch driver's prefetch into the spare slot.  The load then neither counts
// against the logical capacity nor waits for compute work (nothing enqueued uses the spare slot).
int do_swap(legend_ctx* c, int evict, int load, bool fence_now, bool early_load = false) {
    if (evict >= c->n || load >= c->n || evict < -1 || load < -1) return fail(LEGEND_E_INVAL, "partition id out of range");
    if (evict < 0 && load < 0) return LEGEND_OK;
    if (evict >= 0 && c->part_slot[evict] < 0) return fail(LEGEND_E_NOT_RESIDENT, "partition %d is not resident", evict);
    if (load >= 0 && c->part_slot[load] >= 0) return fail(LEGEND_E_STATE, "partition %d is already resident", load);
    const size_t bytes = c->part_floats * sizeof(float);
    if (load >= 0 && evict < 0) {
        int resident = 0;
        for (int p = 0; p < c->n; ++p) resident += c->part_slot[p] >= 0;
        if (resident >= (early_load ? c->nslots : c->cap)) return fail(LEGEND_E_STATE, "no free buffer slot for partition %d", load);
    }
    if (fence_now) {
        HIP_TRY(c, hipEventRecord(c->ev_fence, c->compute));
    }
    int out_slot = -1;
    if (evict >= 0) {
        // write-back: after the compute work enqueued so far (it may still use the partition)
        out_slot = c->part_slot[evict];
        HIP_TRY(c, hipStreamWaitEvent(c->copy_out, c->ev_fence, 0));
        if (c->slot_pending[out_slot]) HIP_TRY(c, hipStreamWaitEvent(c->copy_out, c->slot_ready[out_slot], 0));
        HIP_TRY(c, hipMemcpyAsync(c->host_part[evict], c->slot_mem[out_slot], bytes, hipMemcpyDeviceToHost, c->copy_out));
        HIP_TRY(c, hipEventRecord(c->slot_drained[out_slot], c->copy_out));
        c->slot_draining[out_slot] = 1;
        c->slot_drain_part[out_slot] = evict;
        c->part_slot[evict] = -1;
        c->slot_part[out_slot] = -1;
    }
    if (load >= 0) {
        // into a free slot other than the one being written back when there is one
        int slot = -1;
        for (int sl = 0; sl < c->nslots; ++sl)
            if (c->slot_part[sl] < 0 && sl != out_slot) { slot = sl; break; }
        if (slot < 0) slot = out_slot;
        if (slot < 0) return fail(LEGEND_E_STATE, "no free buffer slot for partition %d", load);
        // the slot's previous tenant must be back on the host; and a load never starts before the
        // compute work enqueued so far is done, so that a caller who asks for the swap after a
        // state's last bucket gets a swap that is not hidden behind that bucket
        if (!early_load) HIP_TRY(c, hipStreamWaitEvent(c->copy, c->ev_fence, 0));
        if (c->slot_draining[slot]) {
            HIP_TRY(c, hipStreamWaitEvent(c->copy, c->slot_drained[slot], 0));
            c->slot_draining[slot] = 0;
        }
        // the host block of a partition that is itself still being written back is not read early
        for (int sl = 0; sl < c->nslots; ++sl)
            if (c->slot_draining[sl] && c->slot_drain_part[sl] == load)
                HIP_TRY(c, hipStreamWaitEvent(c->copy, c->slot_drained[sl], 0));
        HIP_TRY(c, hipMemcpyAsync(c->slot_mem[slot], c->host_part[load], bytes, hipMemcpyHostToDevice, c->copy));
        HIP_TRY(c, hipEventRecord(c->slot_ready[slot], c->copy));
        c->slot_pending[slot] = 1;
        c->part_slot[load] = slot;
        c->slot_part[slot] = load;
    }
    c->part_tables_dirty = true;
    return LEGEND_OK;
}

void free_ctx(legend_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->cfg.device);
    if (c->compute) (void)hipStreamSynchronize(c->compute);
    if (c->copy) (void)hipStreamSynchronize(c->copy);
    if (c->copy_out) { (void)hipStreamSynchronize(c->copy_out); (void)hipStreamDestroy(c->copy_out); }
    for (hipEvent_t e : c->slot_drained) if (e) (void)hipEventDestroy(e);
    for (float* p : c->host_part) if (p) (void)hipHostFree(p);
    for (float* p : c->slot_mem) if (p) (void)hipFree(p);
    for (float* p : c->slot_grad) if (p) (void)hipFree(p);
    if (c->G_rel) (void)hipFree(c->G_rel);
    for (hipEvent_t e : c->slot_ready) if (e) (void)hipEventDestroy(e);
    for (auto& s : c->prof_spans) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
    for (hipEvent_t e : c->prof_pool) (void)hipEventDestroy(e);
    void* frees[] = {c->E_rel, c->S_rel, c->d_part_emb, c->d_part_state, c->ws.neg_ids, c->ws.keys[0], c->ws.keys[1],
                     c->ws.vals[0], c->ws.vals[1], c->ws.ghist, c->ws.scan_tmp, c->ws.uniq_keys, c->ws.seg_start,
                     c->ws.counters, c->ws.long_list, c->ws.unit_start, c->ws.long_partial, c->ws.uniq_total, c->ws.grad, c->ws.loss_partial, c->ws.redo, c->ws.redo_total, c->ws.loss_sum, c->ws.gemm_Q, c->ws.gemm_G, c->ws.gemm_f,
                     c->ws.gemm_a, c->ws.gemm_S, c->edges_dev,
                     c->io_dev};
    for (void* p : frees) if (p) (void)hipFree(p);
    for (Workspace& o : c->ws_alt) {
        void* own[] = {o.neg_ids, o.keys[0], o.keys[1], o.vals[0], o.vals[1], o.ghist, o.scan_tmp, o.uniq_keys, o.seg_start,
                       o.counters, o.long_list, o.unit_start};
        for (void* p : own) if (p) (void)hipFree(p);
    }
    if (c->aux) { (void)hipStreamSynchronize(c->aux); (void)hipStreamDestroy(c->aux); }
    if (c->aux2) { (void)hipStreamSynchronize(c->aux2); (void)hipStreamDestroy(c->aux2); }
    if (c->ev_chunk_done) (void)hipEventDestroy(c->ev_chunk_done);
    if (c->ev_long_done) (void)hipEventDestroy(c->ev_long_done);
    if (c->ev_start) (void)hipEventDestroy(c->ev_start);
    for (int k = 0; k < 3; ++k) {
        if (c->ev_index[k]) (void)hipEventDestroy(c->ev_index[k]);
        if (c->ev_updated[k]) (void)hipEventDestroy(c->ev_updated[k]);
    }
    if (c->ev_fence) (void)hipEventDestroy(c->ev_fence);
    if (c->ev_t0) (void)hipEventDestroy(c->ev_t0);
    if (c->ev_t1) (void)hipEventDestroy(c->ev_t1);
    if (c->own_compute && c->compute) (void)hipStreamDestroy(c->compute);
    if (c->own_copy && c->copy) (void)hipStreamDestroy(c->copy);
    delete c;
}

template <typename T>
int dev_alloc(legend_ctx* c, T** p, size_t count) {
    void* q = nullptr;
    size_t bytes = std::max<size_t>(count, 1) * sizeof(T);
    if (hipMalloc(&q, bytes) != hipSuccess) {
        (void)hipGetLastError();
        (void)c;
        return fail(LEGEND_E_NOMEM, "device allocation of %zu bytes failed", bytes);
    }
    *p = static_cast<T*>(q);
    return LEGEND_OK;
}

int check_ctx(legend_ctx* c) {
    if (!c) return fail(LEGEND_E_INVAL, "null context");
    if (c->fatal) return fail(LEGEND_E_HIP, "context is unusable after an earlier HIP failure");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(LEGEND_E_HIP, "hipSetDevice(%d) failed", c->cfg.device);
    return LEGEND_OK;
}

// Stage a bucket's edges on the device if they are in host memory; validate ids.
int stage_edges(legend_ctx* c, int i, int j, const int32_t* edges, int64_t m, int mem, const int32_t** dev_out) {
    const int32_t* dev = edges;
    if (mem == LEGEND_MEM_HOST) {
        if (m > c->edges_cap) {
            HIP_TRY(c, hipStreamSynchronize(c->compute));
            if (c->edges_dev) HIP_TRY(c, hipFree(c->edges_dev));
            c->edges_dev = nullptr;
            c->edges_cap = 0;
            int64_t want = std::max<int64_t>(m, 1 << 16);
            int rc = dev_alloc(c, &c->edges_dev, (size_t)want * 3);
            if (rc) return rc;
            c->edges_cap = want;
        }
        if (m > 0)
            HIP_TRY(c, hipMemcpyAsync(c->edges_dev, edges, (size_t)m * 3 * sizeof(int32_t), hipMemcpyHostToDevice, c->compute));
        dev = c->edges_dev;
    } else if (mem != LEGEND_MEM_DEVICE) {
        return fail(LEGEND_E_INVAL, "edges_mem must be LEGEND_MEM_HOST or LEGEND_MEM_DEVICE");
    }
    uint32_t* flag = c->ws.counters + 1;
    HIP_TRY(c, hipMemsetAsync(flag, 0, sizeof(uint32_t), c->compute));
    {
        ProfScope ps(c, KC_MISC);
        HIP_TRY(c, launch_validate_edges(c->compute, dev, m, (int32_t)rows_valid(c, i), (int32_t)rows_valid(c, j),
                                         c->cfg.num_relations, c->uses_rel ? 1 : 0, flag));
    }
    uint32_t h = 0;
    HIP_TRY(c, hipMemcpyAsync(&h, flag, sizeof h, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    if (h) return fail(LEGEND_E_RANGE, "bucket (%d,%d) holds a node or relation id outside its table", i, j);
    *dev_out = dev;
    return LEGEND_OK;
}

int bucket_params(legend_ctx* c, int i, int j, const int32_t* dev_edges, int64_t m, BucketParams* bp) {
    int si = c->part_slot[i], sj = c->part_slot[j];
    if (si < 0 || sj < 0) return fail(LEGEND_E_NOT_RESIDENT, "bucket (%d,%d): partition %d is not resident", i, j, si < 0 ? i : j);
    int rc = wait_slot(c, si);
    if (rc) return rc;
    rc = wait_slot(c, sj);
    if (rc) return rc;
    const int64_t half = c->Rp * c->d;
    BucketParams p{};
    p.edges = dev_edges;
    p.m = m;
    p.E_src = c->slot_mem[si]; p.S_src = c->slot_mem[si] + half;
    p.E_dst = c->slot_mem[sj]; p.S_dst = c->slot_mem[sj] + half;
    p.E_rel = c->E_rel; p.S_rel = c->S_rel;
    p.atomic_mode = c->cfg.update_mode == LEGEND_UPDATE_ATOMIC ? 1 : 0;
    p.G_src = c->slot_grad[si]; p.G_dst = c->slot_grad[sj]; p.G_rel = c->G_rel;
    p.rows_valid_src = (int32_t)rows_valid(c, i);
    p.rows_valid_dst = (int32_t)rows_valid(c, j);
    p.num_relations = c->cfg.num_relations;
    p.dim = c->d;
    p.score = c->cfg.score;
    p.loss = c->cfg.loss == LEGEND_LOSS_LOGISTIC ? LEGEND_LOSS_LOGISTIC
             : (c->cfg.loss == LEGEND_LOSS_MARGIN ? LEGEND_LOSS_MARGIN : LEGEND_LOSS_SOFTMAX);
    p.margin = c->cfg.margin;
    p.softmax_with_pos = c->cfg.loss == LEGEND_LOSS_SOFTMAX_POS ? 1 : 0;
    p.same_part = i == j;
    p.key_base_dst = i == j ? 0u : (uint32_t)c->Rp;
    p.key_base_rel = i == j ? (uint32_t)c->Rp : (uint32_t)(2 * c->Rp);
    p.num_degree_negs = c->cfg.num_degree_negs;
    p.lr = c->cfg.lr;
    p.eps = c->cfg.eps;
    p.neg_weight = c->cfg.neg_weight >= 0.f ? c->cfg.neg_weight : 1.0f / (float)c->cfg.num_negs;
    *bp = p;
    return LEGEND_OK;
}

uint64_t batch_hash_prefix(const legend_ctx* c, int epoch, int i, int j, int64_t b) {
    uint64_t h = c->cfg.seed;
    h = hash_fold(h, (uint64_t)(int64_t)epoch);
    h = hash_fold(h, (uint64_t)i);
    h = hash_fold(h, (uint64_t)j);
    h = hash_fold(h, (uint64_t)b);
    return h;
}

// index side of one batch: negatives, keys, sort, segment heads, all on stream `st` into `ws`
int enqueue_index_side(legend_ctx* c, hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws,
                       int* sorted_buf) {
    {
        ProfScope ps(c, KC_PREPARE, st);
        HIP_TRY(c, launch_prepare(st, g, bp, ws));
    }
    {
        ProfScope ps(c, KC_SORT, st);
        const bool plan_long = c->cfg.update_mode != LEGEND_UPDATE_ATOMIC;
        HIP_TRY(c, launch_sort_and_segments(st, g, bp, c->key_bits, ws, sorted_buf, plan_long));
        if (plan_long) HIP_TRY(c, launch_long_plan(st, g.n_occ, ws));
    }
    return LEGEND_OK;
}

}  // namespace

extern "C" {

const char* legend_last_error(void) { return g_last_error; }

const char* legend_profile_name(int32_t k) { return (k >= 0 && k < KC_COUNT) ? kClassNames[k] : nullptr; }

int legend_init_partitions(const legend_config* cfg, const float* init_node_emb, const float* init_rel_emb,
                           legend_ctx** out) {
    return guarded("legend_init_partitions", [&]() -> int {
    if (!cfg || !out) return fail(LEGEND_E_INVAL, "cfg and out must not be NULL");
    *out = nullptr;
    if (cfg->struct_size != sizeof(legend_config))
        return fail(LEGEND_E_INVAL, "legend_config.struct_size is %u, library expects %zu", cfg->struct_size, sizeof(legend_config));
    if (cfg->num_nodes < 1 || cfg->dim < 1 || cfg->num_partitions < 1 || cfg->num_partitions > cfg->num_nodes)
        return fail(LEGEND_E_INVAL, "num_nodes, dim, num_partitions must be positive and num_partitions <= num_nodes");
    if (!dim_supported(cfg->dim))
        return fail(LEGEND_E_INVAL, "dim %d is not supported (1..%d)", cfg->dim, max_dim_supported());
    if (cfg->score < 0 || cfg->score > 3 || cfg->loss < 0 || cfg->loss > 3 || cfg->corrupt < 0 || cfg->corrupt > 2)
        return fail(LEGEND_E_INVAL, "unknown score, loss or corrupt selector");
    if (cfg->loss == LEGEND_LOSS_MARGIN && !(cfg->margin >= 0.f))
        return fail(LEGEND_E_INVAL, "the margin loss needs margin >= 0");
    if (cfg->update_mode != LEGEND_UPDATE_DETERMINISTIC && cfg->update_mode != LEGEND_UPDATE_ATOMIC)
        return fail(LEGEND_E_INVAL, "unknown update_mode %d", cfg->update_mode);
    if (cfg->score == LEGEND_SCORE_COMPLEX && (cfg->dim & 1)) return fail(LEGEND_E_INVAL, "ComplEx needs an even dim");
    if (cfg->score == LEGEND_SCORE_TRANSE_L1 && cfg->dim > 128)
        return fail(LEGEND_E_INVAL, "the translational score is implemented for dim <= 128");
    if (cfg->score != LEGEND_SCORE_DOT && cfg->num_relations < 1)
        return fail(LEGEND_E_INVAL, "this score function needs num_relations >= 1");
    if ((!init_node_emb || (cfg->score != LEGEND_SCORE_DOT && !init_rel_emb)) && !(cfg->init_std > 0.f))
        return fail(LEGEND_E_INVAL, "a NULL initial table asks for the seeded fill, which needs init_std > 0");
    if (cfg->batch_size < 1 || cfg->chunk_size < 1 || cfg->num_negs < 1 || cfg->num_degree_negs < 0 ||
        cfg->num_degree_negs > cfg->num_negs)
        return fail(LEGEND_E_INVAL, "batch_size, chunk_size, num_negs must be >= 1 and 0 <= num_degree_negs <= num_negs");
    if (cfg->buffer_capacity < 1 || cfg->buffer_capacity > cfg->num_partitions)
        return fail(LEGEND_E_INVAL, "buffer_capacity must be in [1, num_partitions]");
    if (!(cfg->lr > 0.f) || !(cfg->eps >= 0.f)) return fail(LEGEND_E_INVAL, "lr must be > 0 and eps >= 0");
    const int64_t Rp = (cfg->num_nodes + cfg->num_partitions - 1) / cfg->num_partitions;
    if ((int64_t)(cfg->num_partitions - 1) * Rp >= cfg->num_nodes)
        return fail(LEGEND_E_INVAL, "num_partitions %d leaves an empty partition for %lld nodes", cfg->num_partitions, (long long)cfg->num_nodes);
    if (2 * Rp + std::max(cfg->num_relations, 1) >= (int64_t)1 << 31) return fail(LEGEND_E_INVAL, "partition too large for 32-bit row keys");

    if (hipSetDevice(cfg->device) != hipSuccess) return fail(LEGEND_E_HIP, "hipSetDevice(%d) failed", cfg->device);
    {
        int rc_scratch = resolve_static_scratch(cfg->device);
        if (rc_scratch) return rc_scratch;
    }
    legend_ctx* c = new (std::nothrow) legend_ctx();
    if (!c) return fail(LEGEND_E_NOMEM, "context allocation failed");
    try {
    c->cfg = *cfg;
    c->V = cfg->num_nodes;
    c->n = cfg->num_partitions;
    c->cap = cfg->buffer_capacity;
    c->d = cfg->dim;
    c->Rp = Rp;
    c->part_floats = (size_t)2 * Rp * c->d;
    c->uses_rel = cfg->score != LEGEND_SCORE_DOT;
    {
        const char* e = std::getenv("LEGEND_SERIAL_SORT");
        c->serial_sort = e && e[0] == '1';
        const char* wc = std::getenv("LEGEND_INDEX_AFTER_CHUNK");
        c->index_after_chunk = wc && wc[0] == '1';
        const char* ns = std::getenv("LEGEND_NO_SMALL_UPDATE");
        c->no_small_update = ns && ns[0] == '1';
    }
    c->nrel_rows = std::max(cfg->num_relations, 1);
    c->host_part.assign(c->n, nullptr);
    c->nslots = c->cap < c->n ? c->cap + 1 : c->cap;
    c->slot_mem.assign(c->nslots, nullptr);
    c->slot_grad.assign(c->nslots, nullptr);
    c->slot_part.assign(c->nslots, -1);
    c->part_slot.assign(c->n, -1);
    c->h_part_emb.assign(c->n, nullptr);
    c->h_part_state.assign(c->n, nullptr);
    c->slot_ready.assign(c->nslots, nullptr);
    c->slot_pending.assign(c->nslots, 0);
    c->slot_drained.assign(c->nslots, nullptr);
    c->slot_draining.assign(c->nslots, 0);
    c->slot_drain_part.assign(c->nslots, -1);

#define INIT_TRY(expr)                                                                                   \
    do {                                                                                                 \
        hipError_t _e = (expr);                                                                          \
        if (_e != hipSuccess) {                                                                          \
            int _rc = fail(_e == hipErrorOutOfMemory ? LEGEND_E_NOMEM : LEGEND_E_HIP, "%s failed: %s", #expr, \
                           hipGetErrorString(_e));                                                       \
            (void)hipGetLastError();                                                                     \
            free_ctx(c);                                                                                 \
            return _rc;                                                                                  \
        }                                                                                                \
    } while (0)
#define INIT_RC(expr)                  \
    do {                               \
        int _rc = (expr);              \
        if (_rc) {                     \
            free_ctx(c);               \
            return _rc;                \
        }                              \
    } while (0)

    if (cfg->compute_stream) c->compute = (hipStream_t)cfg->compute_stream;
    else { INIT_TRY(hipStreamCreateWithFlags(&c->compute, hipStreamNonBlocking)); c->own_compute = true; }
    if (cfg->copy_stream) c->copy = (hipStream_t)cfg->copy_stream;
    else { INIT_TRY(hipStreamCreateWithFlags(&c->copy, hipStreamNonBlocking)); c->own_copy = true; }
    INIT_TRY(hipEventCreateWithFlags(&c->ev_fence, hipEventDisableTiming));
    INIT_TRY(hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking));
    INIT_TRY(hipEventCreateWithFlags(&c->ev_chunk_done, hipEventDisableTiming));
    INIT_TRY(hipEventCreateWithFlags(&c->ev_long_done, hipEventDisableTiming));
    INIT_TRY(hipEventCreateWithFlags(&c->ev_start, hipEventDisableTiming));
    for (int k = 0; k < 3; ++k) {
        INIT_TRY(hipEventCreateWithFlags(&c->ev_index[k], hipEventDisableTiming));
        INIT_TRY(hipEventCreateWithFlags(&c->ev_updated[k], hipEventDisableTiming));
    }
    INIT_TRY(hipEventCreate(&c->ev_t0));
    INIT_TRY(hipEventCreate(&c->ev_t1));
    INIT_TRY(hipEventRecord(c->ev_fence, c->compute));

    // host tier: one pinned block [E_p | S_p] per partition (the paper's contiguous SSD layout)
    const size_t half = (size_t)Rp * c->d;
    for (int p = 0; p < c->n; ++p) {
        void* q = nullptr;
        INIT_TRY(hipHostMalloc(&q, c->part_floats * sizeof(float), hipHostMallocDefault));
        c->host_part[p] = static_cast<float*>(q);
        const int64_t lo = (int64_t)p * Rp;
        const int64_t rows = std::max<int64_t>(0, std::min<int64_t>(Rp, c->V - lo));
        if (init_node_emb) std::memcpy(c->host_part[p], init_node_emb + lo * c->d, (size_t)rows * c->d * sizeof(float));
        std::memset(c->host_part[p] + (size_t)(init_node_emb ? rows : 0) * c->d, 0,
                    (c->part_floats - (size_t)(init_node_emb ? rows : 0) * c->d) * sizeof(float));
        (void)half;
    }
    INIT_TRY(hipStreamCreateWithFlags(&c->copy_out, hipStreamNonBlocking));
    // A process has four hardware queues; a fifth stream shares one with another, and a kernel that
    // shares a queue with a multi-gigabyte partition transfer waits for it.  With a staged buffer the
    // two copy streams are busy and the third compute-side stream stays unused (and is not created).
    if (c->nslots == c->cap) INIT_TRY(hipStreamCreateWithFlags(&c->aux2, hipStreamNonBlocking));
    for (int s = 0; s < c->nslots; ++s) {
        INIT_RC(dev_alloc(c, &c->slot_mem[s], c->part_floats));
        INIT_TRY(hipEventCreateWithFlags(&c->slot_ready[s], hipEventDisableTiming));
        INIT_TRY(hipEventCreateWithFlags(&c->slot_drained[s], hipEventDisableTiming));
        if (cfg->update_mode == LEGEND_UPDATE_ATOMIC) {
            INIT_RC(dev_alloc(c, &c->slot_grad[s], (size_t)Rp * c->d));
            INIT_TRY(hipMemset(c->slot_grad[s], 0, (size_t)Rp * c->d * sizeof(float)));
        }
    }
    if (!init_node_emb) {
        // seeded fill: generated on the device into the first slot, one partition at a time, and copied to the host tier
        for (int p = 0; p < c->n; ++p) {
            const int64_t lo = (int64_t)p * Rp;
            const int64_t rows = std::max<int64_t>(0, std::min<int64_t>(Rp, c->V - lo));
            INIT_TRY(launch_init_fill(c->compute, c->slot_mem[0], rows, c->d, lo, cfg->seed, kInitTagNode, cfg->init_std));
            INIT_TRY(hipMemcpyAsync(c->host_part[p], c->slot_mem[0], (size_t)rows * c->d * sizeof(float), hipMemcpyDeviceToHost, c->compute));
        }
        INIT_TRY(hipStreamSynchronize(c->compute));
    }
    const size_t rel_floats = (size_t)c->nrel_rows * c->d;
    INIT_RC(dev_alloc(c, &c->E_rel, rel_floats));
    INIT_RC(dev_alloc(c, &c->S_rel, rel_floats));
    INIT_TRY(hipMemset(c->S_rel, 0, rel_floats * sizeof(float)));
    if (cfg->update_mode == LEGEND_UPDATE_ATOMIC) {
        INIT_RC(dev_alloc(c, &c->G_rel, rel_floats));
        INIT_TRY(hipMemset(c->G_rel, 0, rel_floats * sizeof(float)));
    }
    if (init_rel_emb) INIT_TRY(hipMemcpy(c->E_rel, init_rel_emb, rel_floats * sizeof(float), hipMemcpyHostToDevice));
    else if (c->uses_rel) INIT_TRY(launch_init_fill(c->compute, c->E_rel, c->nrel_rows, c->d, 0, cfg->seed, kInitTagRel, cfg->init_std));
    else INIT_TRY(hipMemset(c->E_rel, 0, rel_floats * sizeof(float)));
    INIT_RC(dev_alloc(c, &c->d_part_emb, (size_t)c->n));
    INIT_RC(dev_alloc(c, &c->d_part_state, (size_t)c->n));
    INIT_TRY(hipMemset(c->d_part_emb, 0, sizeof(float*) * c->n));
    INIT_TRY(hipMemset(c->d_part_state, 0, sizeof(float*) * c->n));

    // per-batch workspace sized for a full batch
    c->gmax = make_geom(c, cfg->batch_size);
    const int64_t occ = c->gmax.n_occ;
    const int64_t nwg = (int64_t)c->gmax.sides * c->gmax.nchunks * c->gmax.T;
    {
        uint64_t maxkey = (uint64_t)2 * Rp + c->nrel_rows;
        int bits = 1;
        while (bits < 32 && (1ull << bits) <= maxkey) ++bits;
        c->key_bits = bits;
    }
    const int64_t nblk = (occ + 2047) / 2048;
    if (nblk * 256 > (int64_t)2048 * 2048) { free_ctx(c); return fail(LEGEND_E_INVAL, "batch too large for the sorter"); }
    Workspace& w = c->ws;
    w.cap_occ = occ;
    w.cap_wg = nwg;
    INIT_RC(dev_alloc(c, &w.neg_ids, (size_t)c->gmax.sides * c->gmax.nchunks * c->gmax.N));
    for (int k = 0; k < 2; ++k) {
        INIT_RC(dev_alloc(c, &w.keys[k], (size_t)occ));
        INIT_RC(dev_alloc(c, &w.vals[k], (size_t)occ));
    }
    INIT_RC(dev_alloc(c, &w.ghist, (size_t)nblk * 256));
    INIT_RC(dev_alloc(c, &w.scan_tmp, (size_t)std::max<int64_t>(nblk, (nblk * 256 + 2047) / 2048) + 2));
    INIT_RC(dev_alloc(c, &w.uniq_keys, (size_t)occ));
    INIT_RC(dev_alloc(c, &w.seg_start, (size_t)occ + 1));
    INIT_RC(dev_alloc(c, &w.counters, 8));
    INIT_RC(dev_alloc(c, &w.long_list, (size_t)update_long_rows_capacity(occ)));
    INIT_RC(dev_alloc(c, &w.unit_start, (size_t)update_long_rows_capacity(occ) + 1));
    INIT_RC(dev_alloc(c, &w.long_partial, (size_t)update_long_units_capacity(occ) * c->d));
    INIT_RC(dev_alloc(c, &w.uniq_total, 1));
    INIT_RC(dev_alloc(c, &w.grad, (size_t)occ * c->d));
    INIT_RC(dev_alloc(c, &w.loss_partial, (size_t)nwg));
    INIT_RC(dev_alloc(c, &w.redo, (size_t)nwg));
    INIT_RC(dev_alloc(c, &w.redo_total, 1));
    INIT_TRY(hipMemset(w.redo_total, 0, sizeof(unsigned long long)));
    {
        const char* e = std::getenv("LEGEND_NO_FAST_CHUNK");
        w.no_fast_path = (e && e[0] == '1') ? 1 : 0;
        const char* nr = std::getenv("LEGEND_FAST_CHUNK_NO_RESCALE");
        w.fast_no_rescale = (nr && nr[0] == '1') ? 1 : 0;
        const char* lim = std::getenv("LEGEND_FAST_CHUNK_LIMIT");
        w.fast_limit = lim ? (float)std::atof(lim) : 110.f;
        if (!(w.fast_limit <= 110.f)) w.fast_limit = 110.f;   // a test knob: it can only tighten the limit
    }
    INIT_RC(dev_alloc(c, &w.loss_sum, 1));
    if (c->d > 128) {
        const size_t rows = (size_t)c->gmax.sides * cfg->batch_size;
        INIT_RC(dev_alloc(c, &w.gemm_Q, rows * c->d));
        INIT_RC(dev_alloc(c, &w.gemm_G, rows * c->d));
        INIT_RC(dev_alloc(c, &w.gemm_f, rows));
        INIT_RC(dev_alloc(c, &w.gemm_a, rows));
        INIT_RC(dev_alloc(c, &w.gemm_S, (size_t)nwg * c->gmax.rows_tile * (size_t)gemm_npad(c->gmax.N)));
    }
    // Two more sets of index-side buffers: the index side of batch b+1 is built while batch b is still
    // being computed and applied, into the set that batch b-2 has released (so it does not wait for
    // the update of batch b-1 either).
    for (Workspace& o : c->ws_alt) {
        o = w;
        o.neg_ids = nullptr; o.keys[0] = o.keys[1] = nullptr; o.vals[0] = o.vals[1] = nullptr;
        o.ghist = nullptr; o.scan_tmp = nullptr; o.uniq_keys = nullptr; o.seg_start = nullptr; o.counters = nullptr;
        o.long_list = nullptr; o.unit_start = nullptr;
        INIT_RC(dev_alloc(c, &o.long_list, (size_t)update_long_rows_capacity(occ)));
        INIT_RC(dev_alloc(c, &o.unit_start, (size_t)update_long_rows_capacity(occ) + 1));
        INIT_RC(dev_alloc(c, &o.neg_ids, (size_t)c->gmax.sides * c->gmax.nchunks * c->gmax.N));
        for (int k = 0; k < 2; ++k) {
            INIT_RC(dev_alloc(c, &o.keys[k], (size_t)occ));
            INIT_RC(dev_alloc(c, &o.vals[k], (size_t)occ));
        }
        INIT_RC(dev_alloc(c, &o.ghist, (size_t)nblk * 256));
        INIT_RC(dev_alloc(c, &o.scan_tmp, (size_t)std::max<int64_t>(nblk, (nblk * 256 + 2047) / 2048) + 2));
        INIT_RC(dev_alloc(c, &o.uniq_keys, (size_t)occ));
        INIT_RC(dev_alloc(c, &o.seg_start, (size_t)occ + 1));
        INIT_RC(dev_alloc(c, &o.counters, 8));
        INIT_TRY(hipMemset(o.counters, 0, 8 * sizeof(uint32_t)));
    }
    INIT_TRY(hipMemset(w.counters, 0, 8 * sizeof(uint32_t)));
    INIT_TRY(hipMemset(w.uniq_total, 0, sizeof(unsigned long long)));
    INIT_TRY(hipMemset(w.loss_sum, 0, sizeof(double)));
    INIT_TRY(hipDeviceSynchronize());
#undef INIT_TRY
#undef INIT_RC
    } catch (...) {
        free_ctx(c);
        throw;
    }
    *out = c;
    return LEGEND_OK;
    });
}

int legend_destroy(legend_ctx* ctx) {
    return guarded("legend_destroy", [&]() -> int {
    free_ctx(ctx);
    return LEGEND_OK;
    });
}

int legend_sync(legend_ctx* c) {
    return guarded("legend_sync", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    if (c->aux2) HIP_TRY(c, hipStreamSynchronize(c->aux2));
    HIP_TRY(c, hipStreamSynchronize(c->copy));
    HIP_TRY(c, hipStreamSynchronize(c->copy_out));
    return LEGEND_OK;
    });
}

int legend_swap_partition(legend_ctx* c, int32_t evict, int32_t load) {
    return guarded("legend_swap_partition", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    return do_swap(c, evict, load, true);
    });
}

int legend_partition_slot(legend_ctx* c, int32_t part, int32_t* slot) {
    return guarded("legend_partition_slot", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!slot || part < 0 || part >= c->n) return fail(LEGEND_E_INVAL, "bad partition id or NULL output");
    *slot = c->part_slot[part];
    return LEGEND_OK;
    });
}

int legend_train_bucket(legend_ctx* c, int32_t i, int32_t j, const int32_t* edges, int64_t m, int32_t edges_mem,
                        int32_t epoch, const legend_prefetch* hint, legend_bucket_stats* stats) {
    return guarded("legend_train_bucket", [&]() -> int {
    return legend_train_bucket_range(c, i, j, edges, m, edges_mem, epoch, 0, -1, hint, stats);
    });
}

int legend_train_bucket_range(legend_ctx* c, int32_t i, int32_t j, const int32_t* edges, int64_t m, int32_t edges_mem,
                              int32_t epoch, int64_t batch_begin, int64_t batch_end, const legend_prefetch* hint,
                              legend_bucket_stats* stats) {
    return guarded("legend_train_bucket_range", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (i < 0 || j < 0 || i >= c->n || j >= c->n) return fail(LEGEND_E_INVAL, "bucket (%d,%d) out of range", i, j);
    if (m < 0 || (m > 0 && !edges)) return fail(LEGEND_E_INVAL, "edges must not be NULL when m > 0");
    {
        const int64_t nb_all = (m + c->cfg.batch_size - 1) / c->cfg.batch_size;
        if (batch_end < 0) batch_end = nb_all;
        if (batch_begin < 0 || batch_begin > batch_end || batch_end > nb_all)
            return fail(LEGEND_E_INVAL, "batch range [%lld, %lld) outside [0, %lld]", (long long)batch_begin,
                        (long long)batch_end, (long long)nb_all);
    }
    if (c->part_slot[i] < 0 || c->part_slot[j] < 0)
        return fail(LEGEND_E_NOT_RESIDENT, "bucket (%d,%d): partition %d is not resident", i, j, c->part_slot[i] < 0 ? i : j);
    if (hint) {
        if (hint->evict >= c->n || hint->load >= c->n || hint->evict < -1 || hint->load < -1)
            return fail(LEGEND_E_INVAL, "prefetch hint out of range");
        if (hint->evict >= 0 && c->part_slot[hint->evict] < 0)
            return fail(LEGEND_E_NOT_RESIDENT, "prefetch hint evicts partition %d which is not resident", hint->evict);
        if (hint->load >= 0 && c->part_slot[hint->load] >= 0)
            return fail(LEGEND_E_STATE, "prefetch hint loads partition %d which is already resident", hint->load);
    }
    const int32_t* dev_edges = nullptr;
    BucketParams bp{};
    rc = bucket_params(c, i, j, nullptr, m, &bp);
    if (rc) return rc;
    rc = stage_edges(c, i, j, edges, m, edges_mem, &dev_edges);
    if (rc) return rc;
    bp.edges = dev_edges;

    // a swap that does not touch this bucket may run while the bucket trains
    const bool overlap = hint && hint->evict != i && hint->evict != j;
    if (overlap) {
        rc = do_swap(c, hint->evict, hint->load, true);
        if (rc) return rc;
    }
    if (!c->keep_loss) HIP_TRY(c, hipMemsetAsync(c->ws.loss_sum, 0, sizeof(double), c->compute));
    if (stats) HIP_TRY(c, hipEventRecord(c->ev_t0, c->compute));
    const int B = c->cfg.batch_size;
    const int64_t nb = batch_end - batch_begin;
    int64_t edges_done = 0;
    // The index side of a batch (negative ids, sort keys, sort, segment heads) depends on the edge
    // list and the counter hash only.  It is built one batch ahead on the auxiliary stream, into
    // the workspace the batch before last has released, while the compute stream runs the chunk
    // and update kernels of the current batch.
    auto batch_params = [&](int64_t b, BatchGeom* g) {
        const int P = (int)std::min<int64_t>(B, m - b * B);
        *g = make_geom(c, P);
        bp.batch_lo = b * B;
        bp.hash_prefix = batch_hash_prefix(c, epoch, i, j, b);
    };
    int sorted_of[3] = {0, 0, 0};
    auto wset = [&](int k) -> const Workspace& { return k == 0 ? c->ws : c->ws_alt[k - 1]; };
    const bool ahead = !c->serial_sort;
    if (ahead && batch_begin < batch_end) {
        BatchGeom g0;
        batch_params(batch_begin, &g0);
        HIP_TRY(c, hipEventRecord(c->ev_start, c->compute));        // edges staged, earlier calls done with the workspaces
        HIP_TRY(c, hipStreamWaitEvent(c->aux, c->ev_start, 0));
        rc = enqueue_index_side(c, c->aux, g0, bp, c->ws, &sorted_of[0]);
        if (rc) return rc;
        HIP_TRY(c, hipEventRecord(c->ev_index[0], c->aux));
    }
    for (int64_t b = batch_begin; b < batch_end; ++b) {
        const int cur = ahead ? (int)((b - batch_begin) % 3) : 0;
        const Workspace& ws = wset(cur);
        BatchGeom g;
        batch_params(b, &g);
        edges_done += g.P;
        if (ahead) {
            HIP_TRY(c, hipStreamWaitEvent(c->compute, c->ev_index[cur], 0));
        } else {
            rc = enqueue_index_side(c, c->compute, g, bp, ws, &sorted_of[0]);
            if (rc) return rc;
        }
        {
            ProfScope ps(c, KC_CHUNK);
            HIP_TRY(c, launch_chunks(c->compute, g, bp, ws, false));
        }
        if (chunks_use_single_sweep(g, bp, ws)) {
            ProfScope ps(c, KC_CHUNK_REDO);
            HIP_TRY(c, launch_chunks(c->compute, g, bp, ws, true));
        }
        // The table rows with many gradient rows are disjoint from the others: their two-level sums (and
        // the sum of the workgroups' loss terms) run next to the main update kernel, on a third stream
        // where the process has a hardware queue to spare for it, else on the index stream behind the
        // next batch's index side (which ends well inside the update).  A batch of a few thousand gradient rows is bound by launch latency: it
        // stays on one stream, where a kernel follows the other without a hop between streams.
        const bool aside = ahead && !bp.atomic_mode && g.n_occ > 65536;
        hipStream_t ls = !aside ? c->compute : c->aux2 ? c->aux2 : c->aux;
        // ... and a batch of at most a few thousand has its loss sum and its whole update in one launch
        const bool small = !bp.atomic_mode && !c->no_small_update && update_is_small(g);
        const int64_t loss_terms = (int64_t)g.sides * g.nchunks * g.T;
        if (!aside && !small) {
            ProfScope ps(c, KC_MISC);
            HIP_TRY(c, launch_loss_reduce(c->compute, loss_terms, ws));
        }
        if (aside) HIP_TRY(c, hipEventRecord(c->ev_chunk_done, c->compute));
        if (ahead && b + 1 < batch_end) {
            // next batch's index side: its buffers are free once the update of batch b-2 is done
            const int nxt = (cur + 1) % 3;
            BatchGeom gn;
            BucketParams keep = bp;
            batch_params(b + 1, &gn);
            if (b - batch_begin >= 2) HIP_TRY(c, hipStreamWaitEvent(c->aux, c->ev_updated[nxt], 0));
            if (c->index_after_chunk) {
                if (!aside) HIP_TRY(c, hipEventRecord(c->ev_chunk_done, c->compute));
                HIP_TRY(c, hipStreamWaitEvent(c->aux, c->ev_chunk_done, 0));
            }
            rc = enqueue_index_side(c, c->aux, gn, bp, wset(nxt), &sorted_of[nxt]);
            if (rc) return rc;
            HIP_TRY(c, hipEventRecord(c->ev_index[nxt], c->aux));
            bp = keep;
        }
        if (bp.atomic_mode) {
            ProfScope ps(c, KC_UPDATE);
            HIP_TRY(c, launch_update_atomic(c->compute, g, bp, ws));
        } else if (small) {
            ProfScope ps(c, KC_UPDATE);
            HIP_TRY(c, launch_update_small(c->compute, g, bp, ws, ws.vals[sorted_of[cur]], loss_terms));
        } else {
            if (aside) {
                HIP_TRY(c, hipStreamWaitEvent(ls, c->ev_chunk_done, 0));
                ProfScope ps(c, KC_MISC, ls);
                HIP_TRY(c, launch_loss_reduce(ls, loss_terms, ws));
            }
            {
                ProfScope ps(c, KC_UPDATE_LONG, ls);
                HIP_TRY(c, launch_update(ls, g, bp, ws, ws.vals[sorted_of[cur]], true));
            }
            if (aside) HIP_TRY(c, hipEventRecord(c->ev_long_done, ls));
            {
                ProfScope ps(c, KC_UPDATE);
                HIP_TRY(c, launch_update(c->compute, g, bp, ws, ws.vals[sorted_of[cur]], false));
            }
            if (aside) HIP_TRY(c, hipStreamWaitEvent(c->compute, c->ev_long_done, 0));
        }
        if (ahead) HIP_TRY(c, hipEventRecord(c->ev_updated[cur], c->compute));
        c->batches_done += 1;
    }
    if (stats) HIP_TRY(c, hipEventRecord(c->ev_t1, c->compute));
    if (hint && !overlap) {
        rc = do_swap(c, hint->evict, hint->load, true);
        if (rc) return rc;
    }
    if (stats) {
        double loss = 0.0;
        HIP_TRY(c, hipMemcpyAsync(&loss, c->ws.loss_sum, sizeof loss, hipMemcpyDeviceToHost, c->compute));
        HIP_TRY(c, hipStreamSynchronize(c->compute));
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, c->ev_t0, c->ev_t1));
        stats->loss_sum = loss;
        stats->batches = nb;
        stats->edges = edges_done;
        stats->ms = ms;
    }
    return LEGEND_OK;
    });
}

int legend_train_epoch(legend_ctx* c, const int32_t* const* bucket_edges, const int64_t* bucket_sizes, int32_t edges_mem,
                       int32_t epoch, int32_t overlap, legend_epoch_stats* stats) {
    return guarded("legend_train_epoch", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!bucket_edges || !bucket_sizes) return fail(LEGEND_E_INVAL, "NULL bucket table");
    const int n = c->n;
    for (int b = 0; b < n * n; ++b)
        if (bucket_sizes[b] < 0 || (bucket_sizes[b] > 0 && !bucket_edges[b])) return fail(LEGEND_E_INVAL, "bucket %d: bad size or NULL edges", b);
    if (c->cap < n && (c->cap != 3 || n <= 3))
        return fail(LEGEND_E_INVAL, "an epoch needs buffer_capacity == num_partitions, or 3 with more than 3 partitions");

    // plan: buffer states and bucket order (Sec. 4); with everything resident there is one state
    std::vector<int32_t> states, buckets((size_t)n * n * 2), begin, over;
    int32_t ns = 0;
    {
        int32_t cap_states = 8 * n * n + 8;
        states.resize((size_t)cap_states * 3);
        begin.resize(cap_states + 1);
        over.resize(cap_states);
        rc = legend_plan_order(n, states.data(), cap_states, &ns, buckets.data(), begin.data(), over.data());
        if (rc) return fail(rc, "legend_plan_order failed");
    }
    const bool all_resident = c->cap >= n;
    auto t_begin = std::chrono::steady_clock::now();
    int64_t swaps = 0, edges = 0, batches = 0;

    // bring the first state (or everything) into the buffer
    std::vector<char> want(n, 0);
    if (all_resident) std::fill(want.begin(), want.end(), 1);
    else for (int s = 0; s < 3; ++s) if (states[s] >= 0) want[states[s]] = 1;
    for (int p = 0; p < n; ++p)
        if (!want[p] && c->part_slot[p] >= 0) { rc = do_swap(c, p, -1, true); if (rc) return rc; ++swaps; }
    for (int p = 0; p < n; ++p)
        if (want[p] && c->part_slot[p] < 0) { rc = do_swap(c, -1, p, true); if (rc) return rc; ++swaps; }

    HIP_TRY(c, hipMemsetAsync(c->ws.loss_sum, 0, sizeof(double), c->compute));
    c->keep_loss = true;
    auto train = [&](int idx) -> int {
        const int i = buckets[2 * idx], j = buckets[2 * idx + 1];
        const int64_t m = bucket_sizes[i * n + j];
        if (m == 0) return LEGEND_OK;
        int r = legend_train_bucket_range(c, i, j, bucket_edges[i * n + j], m, edges_mem, epoch, 0, -1, nullptr, nullptr);
        if (r == LEGEND_OK) { edges += m; batches += (m + c->cfg.batch_size - 1) / c->cfg.batch_size; }
        return r;
    };
    rc = LEGEND_OK;
    for (int k = 0; k < ns && rc == LEGEND_OK; ++k) {
        int evict = -1, load = -1;
        if (!all_resident && k + 1 < ns)
            for (int s = 0; s < 3; ++s)
                if (states[3 * k + s] != states[3 * (k + 1) + s]) { evict = states[3 * k + s]; load = states[3 * (k + 1) + s]; }
        // With prefetching and a spare slot the next state's partition starts loading right away: no
        // bucket of this state touches it or the slot it goes to.
        const bool early = overlap && load >= 0 && c->nslots > c->cap;
        if (early) { rc = do_swap(c, -1, load, true, true); if (rc) break; }
        // buckets that involve the partition evicted next
        for (int idx = begin[k]; idx < over[k] && rc == LEGEND_OK; ++idx) rc = train(idx);
        if (rc) break;
        // with prefetching the swap starts now and runs while the remaining buckets train (Sec. 4);
        // without, it starts after them and the next state waits for it
        if (evict >= 0 && overlap) { rc = do_swap(c, evict, early ? -1 : load, true); if (rc) break; ++swaps; }
        for (int idx = over[k]; idx < begin[k + 1] && rc == LEGEND_OK; ++idx) rc = train(idx);
        if (rc) break;
        if (evict >= 0 && !overlap) { rc = do_swap(c, evict, load, true); if (rc) break; ++swaps; }
    }
    c->keep_loss = false;
    if (rc) return rc;
    double loss = 0.0;
    HIP_TRY(c, hipMemcpyAsync(&loss, c->ws.loss_sum, sizeof loss, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->copy));
    HIP_TRY(c, hipStreamSynchronize(c->copy_out));
    if (stats) {
        stats->loss_sum = loss;
        stats->edges = edges;
        stats->batches = batches;
        stats->swaps = swaps;
        stats->buffer_states = all_resident ? 1 : ns;
        stats->bytes_per_swap = (int64_t)(c->part_floats * sizeof(float));
        stats->ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_begin).count();
    }
    return LEGEND_OK;
    });
}

int legend_debug_batch_indices(legend_ctx* c, int32_t i, int32_t j, const int32_t* edges, int64_t m, int32_t edges_mem,
                               int32_t epoch, int64_t batch, int32_t* neg_ids, int64_t neg_capacity, int64_t* touched,
                               int64_t touched_capacity, int64_t* touched_count) {
    return guarded("legend_debug_batch_indices", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (i < 0 || j < 0 || i >= c->n || j >= c->n) return fail(LEGEND_E_INVAL, "bucket (%d,%d) out of range", i, j);
    if (m <= 0 || !edges || !neg_ids || !touched || !touched_count) return fail(LEGEND_E_INVAL, "NULL argument or empty bucket");
    const int B = c->cfg.batch_size;
    const int64_t nb = (m + B - 1) / B;
    if (batch < 0 || batch >= nb) return fail(LEGEND_E_INVAL, "batch %lld out of range (bucket has %lld)", (long long)batch, (long long)nb);
    BucketParams bp{};
    rc = bucket_params(c, i, j, nullptr, m, &bp);
    if (rc) return rc;
    const int32_t* dev_edges = nullptr;
    rc = stage_edges(c, i, j, edges, m, edges_mem, &dev_edges);
    if (rc) return rc;
    bp.edges = dev_edges;
    const int P = (int)std::min<int64_t>(B, m - batch * B);
    BatchGeom g = make_geom(c, P);
    const int64_t nneg = (int64_t)g.sides * g.nchunks * g.N;
    if (neg_capacity < nneg) return fail(LEGEND_E_INVAL, "neg_capacity %lld < %lld", (long long)neg_capacity, (long long)nneg);
    bp.batch_lo = batch * B;
    bp.hash_prefix = batch_hash_prefix(c, epoch, i, j, batch);
    int sorted = 0;
    // the unique-row statistic must not count this dry run
    unsigned long long saved = 0;
    HIP_TRY(c, hipMemcpyAsync(&saved, c->ws.uniq_total, sizeof saved, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    rc = enqueue_index_side(c, c->compute, g, bp, c->ws, &sorted);
    if (rc) return rc;
    uint32_t nu = 0;
    HIP_TRY(c, hipMemcpyAsync(&nu, c->ws.counters, sizeof nu, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipMemcpyAsync(neg_ids, c->ws.neg_ids, (size_t)nneg * sizeof(int32_t), hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipMemcpyAsync(c->ws.uniq_total, &saved, sizeof saved, hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    *touched_count = nu;
    if ((int64_t)nu > touched_capacity) return fail(LEGEND_E_INVAL, "touched_capacity %lld < %u", (long long)touched_capacity, nu);
    std::vector<uint32_t> keys(nu);
    if (nu) HIP_TRY(c, hipMemcpy(keys.data(), c->ws.uniq_keys, (size_t)nu * sizeof(uint32_t), hipMemcpyDeviceToHost));
    for (uint32_t k = 0; k < nu; ++k) {
        uint32_t key = keys[k];
        int64_t t, row;
        if (key >= bp.key_base_rel) { t = 2; row = key - bp.key_base_rel; }
        else if (bp.key_base_dst > 0 && key >= bp.key_base_dst) { t = 1; row = key - bp.key_base_dst; }
        else { t = 0; row = key; }
        touched[k] = (t << 32) + row;
    }
    return LEGEND_OK;
    });
}

int legend_score_edges(legend_ctx* c, const int64_t* src, const int32_t* rel, const int64_t* dst, int64_t m, float* out) {
    return guarded("legend_score_edges", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (m < 0) return fail(LEGEND_E_INVAL, "m < 0");
    if (m == 0) return LEGEND_OK;
    if (!src || !dst || !out) return fail(LEGEND_E_INVAL, "NULL argument");
    if (c->uses_rel && !rel) return fail(LEGEND_E_INVAL, "rel must not be NULL for this score");
    for (int s = 0; s < c->nslots; ++s) {
        rc = wait_slot(c, s);
        if (rc) return rc;
    }
    if (c->part_tables_dirty) {
        rc = upload_part_tables(c);
        if (rc) return rc;
    }
    const size_t b_ids = (size_t)m * sizeof(int64_t), b_rel = (size_t)m * sizeof(int32_t), b_out = (size_t)m * sizeof(float);
    rc = ensure_io(c, 2 * b_ids + b_rel + b_out + 64);
    if (rc) return rc;
    char* base = static_cast<char*>(c->io_dev);
    int64_t* d_src = reinterpret_cast<int64_t*>(base);
    int64_t* d_dst = reinterpret_cast<int64_t*>(base + b_ids);
    float* d_out = reinterpret_cast<float*>(base + 2 * b_ids);
    int32_t* d_rel = reinterpret_cast<int32_t*>(base + 2 * b_ids + b_out);
    uint32_t* flag = c->ws.counters + 1;
    HIP_TRY(c, hipMemsetAsync(flag, 0, sizeof(uint32_t), c->compute));
    HIP_TRY(c, hipMemcpyAsync(d_src, src, b_ids, hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, hipMemcpyAsync(d_dst, dst, b_ids, hipMemcpyHostToDevice, c->compute));
    if (rel) HIP_TRY(c, hipMemcpyAsync(d_rel, rel, b_rel, hipMemcpyHostToDevice, c->compute));
    {
        ProfScope ps(c, KC_MISC);
        HIP_TRY(c, launch_score(c->compute, d_src, rel ? d_rel : nullptr, d_dst, m, c->d_part_emb, (int32_t)c->Rp, c->n,
                                c->V, c->E_rel, c->cfg.num_relations, c->d, c->cfg.score, d_out, flag));
    }
    uint32_t h = 0;
    HIP_TRY(c, hipMemcpyAsync(&h, flag, sizeof h, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipMemcpyAsync(out, d_out, b_out, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    if (h & 1u) return fail(LEGEND_E_RANGE, "a node or relation id is out of range");
    if (h & 2u) return fail(LEGEND_E_NOT_RESIDENT, "an edge refers to a partition that is not resident");
    return LEGEND_OK;
    });
}

int legend_rank_edges(legend_ctx* c, const int64_t* src, const int32_t* rel, const int64_t* dst, int64_t m, int32_t side,
                      const int64_t* candidates, int64_t num_candidates, int32_t* greater, int32_t* equal,
                      legend_rank_metrics* metrics) {
    return guarded("legend_rank_edges", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (m < 0 || num_candidates < 0) return fail(LEGEND_E_INVAL, "m < 0 or num_candidates < 0");
    if (side != LEGEND_CORRUPT_DST && side != LEGEND_CORRUPT_SRC)
        return fail(LEGEND_E_INVAL, "side must be LEGEND_CORRUPT_DST or LEGEND_CORRUPT_SRC");
    if (c->V > 0x7fffffffll) return fail(LEGEND_E_INVAL, "ranking needs num_nodes < 2^31");
    if (metrics) *metrics = legend_rank_metrics{};
    if (m == 0) return LEGEND_OK;
    if (!src || !dst) return fail(LEGEND_E_INVAL, "NULL argument");
    if (c->uses_rel && !rel) return fail(LEGEND_E_INVAL, "rel must not be NULL for this score");
    const int64_t n_cand = candidates ? num_candidates : c->V;
    if (n_cand > 0x7fffffffll) return fail(LEGEND_E_INVAL, "too many candidates");
    for (int s = 0; s < c->nslots; ++s) {
        rc = wait_slot(c, s);
        if (rc) return rc;
    }
    if (c->part_tables_dirty) {
        rc = upload_part_tables(c);
        if (rc) return rc;
    }
    const int64_t m_pad = rank_rows_padded(m);
    const int dp = rank_dim_padded(c->d);
    auto up = [](size_t b) { return (b + 255) & ~(size_t)255; };
    const size_t b_ids = up((size_t)m * sizeof(int64_t)), b_rel = up((size_t)m * sizeof(int32_t));
    const size_t b_cand = up(candidates ? (size_t)n_cand * sizeof(int64_t) : 0);
    const size_t b_q = up((size_t)m_pad * dp * sizeof(float)), b_row = up((size_t)m_pad * sizeof(int32_t));
    rc = ensure_io(c, 2 * b_ids + b_rel + b_cand + b_q + 4 * b_row + 256);
    if (rc) return rc;
    char* p = static_cast<char*>(c->io_dev);
    int64_t* d_src = reinterpret_cast<int64_t*>(p); p += b_ids;
    int64_t* d_dst = reinterpret_cast<int64_t*>(p); p += b_ids;
    int64_t* d_cand = reinterpret_cast<int64_t*>(p); p += b_cand;
    float* d_q = reinterpret_cast<float*>(p); p += b_q;
    float* d_f = reinterpret_cast<float*>(p); p += b_row;
    int32_t* d_true = reinterpret_cast<int32_t*>(p); p += b_row;
    int32_t* d_gt = reinterpret_cast<int32_t*>(p); p += b_row;
    int32_t* d_eq = reinterpret_cast<int32_t*>(p); p += b_row;
    int32_t* d_rel = reinterpret_cast<int32_t*>(p); p += b_rel;
    double* d_metrics = reinterpret_cast<double*>(p);
    uint32_t* flag = c->ws.counters + 1;
    HIP_TRY(c, hipMemsetAsync(flag, 0, sizeof(uint32_t), c->compute));
    HIP_TRY(c, hipMemsetAsync(d_gt, 0, 2 * b_row, c->compute));       // greater and equal are adjacent
    HIP_TRY(c, hipMemcpyAsync(d_src, src, (size_t)m * sizeof(int64_t), hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, hipMemcpyAsync(d_dst, dst, (size_t)m * sizeof(int64_t), hipMemcpyHostToDevice, c->compute));
    if (rel) HIP_TRY(c, hipMemcpyAsync(d_rel, rel, (size_t)m * sizeof(int32_t), hipMemcpyHostToDevice, c->compute));
    if (candidates && n_cand > 0)
        HIP_TRY(c, hipMemcpyAsync(d_cand, candidates, (size_t)n_cand * sizeof(int64_t), hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, hipEventRecord(c->ev_t0, c->compute));
    {
        ProfScope ps(c, KC_MISC);
        HIP_TRY(c, launch_rank(c->compute, d_src, rel ? d_rel : nullptr, d_dst, m, side, candidates ? d_cand : nullptr, n_cand,
                               c->d_part_emb, (int32_t)c->Rp, c->V, c->E_rel, c->cfg.num_relations, c->d, c->cfg.score,
                               d_q, d_f, d_true, d_gt, d_eq, d_metrics, flag));
    }
    HIP_TRY(c, hipEventRecord(c->ev_t1, c->compute));
    uint32_t h = 0;
    double mt[4] = {0, 0, 0, 0};
    HIP_TRY(c, hipMemcpyAsync(&h, flag, sizeof h, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipMemcpyAsync(mt, d_metrics, sizeof mt, hipMemcpyDeviceToHost, c->compute));
    if (greater) HIP_TRY(c, hipMemcpyAsync(greater, d_gt, (size_t)m * sizeof(int32_t), hipMemcpyDeviceToHost, c->compute));
    if (equal) HIP_TRY(c, hipMemcpyAsync(equal, d_eq, (size_t)m * sizeof(int32_t), hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    if (h & 1u) return fail(LEGEND_E_RANGE, "a node, relation or candidate id is out of range");
    if (h & 2u) return fail(LEGEND_E_NOT_RESIDENT, "a triple or a candidate refers to a partition that is not resident");
    if (metrics) {
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, c->ev_t0, c->ev_t1));
        metrics->mrr = mt[0]; metrics->hits1 = mt[1]; metrics->hits3 = mt[2]; metrics->hits10 = mt[3];
        metrics->ms = ms;
    }
    return LEGEND_OK;
    });
}

int legend_rank_edges_static(legend_ctx* c, const int64_t* src, const int32_t* rel, const int64_t* dst, int64_t m,
                             int32_t side, const int64_t* candidates, int64_t num_candidates, int32_t* greater,
                             int32_t* equal, double* metrics, uint32_t* status) {
    return guarded("legend_rank_edges_static", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (m < 0 || num_candidates < 0) return fail(LEGEND_E_INVAL, "m < 0 or num_candidates < 0");
    if (side != LEGEND_CORRUPT_DST && side != LEGEND_CORRUPT_SRC)
        return fail(LEGEND_E_INVAL, "side must be LEGEND_CORRUPT_DST or LEGEND_CORRUPT_SRC");
    if (c->V > 0x7fffffffll) return fail(LEGEND_E_INVAL, "ranking needs num_nodes < 2^31");
    if (!metrics || !status) return fail(LEGEND_E_INVAL, "metrics and status must not be NULL");
    if (m > 0 && (!src || !dst || !greater || !equal)) return fail(LEGEND_E_INVAL, "NULL argument");
    if (m > 0 && c->uses_rel && !rel) return fail(LEGEND_E_INVAL, "rel must not be NULL for this score");
    const int64_t n_cand = candidates ? num_candidates : c->V;
    if (n_cand > 0x7fffffffll) return fail(LEGEND_E_INVAL, "too many candidates");
    // scratch layout: q rows [m_pad][dp] | own scores [m_pad] | true endpoints [m_pad]
    const int64_t m_pad = rank_rows_padded(std::max<int64_t>(m, 1));
    const int dp = rank_dim_padded(c->d);
    auto up = [](size_t b) { return (b + 255) & ~(size_t)255; };
    const size_t b_q = up((size_t)m_pad * dp * sizeof(float)), b_row = up((size_t)m_pad * sizeof(int32_t));
    if (b_q + 2 * b_row > kStaticScratchBytes)
        return fail(LEGEND_E_INVAL, "%lld triples of dimension %d need %zu bytes of scratch, the static buffer holds %zu "
                    "(at most %lld triples at this dimension)", (long long)m, c->d, b_q + 2 * b_row, kStaticScratchBytes,
                    (long long)legend_rank_edges_static_max_triples(c->d));
    unsigned char* base = g_static_scratch[c->cfg.device];
    if (!base) return fail(LEGEND_E_STATE, "static scratch of device %d was never resolved", c->cfg.device);
    for (int s = 0; s < c->nslots; ++s) {
        rc = wait_slot(c, s);
        if (rc) return rc;
    }
    if (c->part_tables_dirty) {
        rc = upload_part_tables(c);
        if (rc) return rc;
    }
    float* d_q = reinterpret_cast<float*>(base);
    float* d_f = reinterpret_cast<float*>(base + b_q);
    int32_t* d_true = reinterpret_cast<int32_t*>(base + b_q + b_row);
    // counts and the status word start at zero; a fill kernel, not a memset node, so that the call can be
    // recorded into a graph
    HIP_TRY(c, launch_fill_u32(c->compute, reinterpret_cast<uint32_t*>(greater), 0u, m));
    HIP_TRY(c, launch_fill_u32(c->compute, reinterpret_cast<uint32_t*>(equal), 0u, m));
    HIP_TRY(c, launch_fill_u32(c->compute, status, 0u, 1));
    HIP_TRY(c, launch_fill_u32(c->compute, reinterpret_cast<uint32_t*>(metrics), 0u, 8));
    if (m == 0) return LEGEND_OK;
    // no event-timed profiling span here: creating its events would allocate
    HIP_TRY(c, launch_rank(c->compute, src, rel, dst, m, side, candidates, n_cand, c->d_part_emb, (int32_t)c->Rp, c->V,
                           c->E_rel, c->cfg.num_relations, c->d, c->cfg.score, d_q, d_f, d_true, greater, equal,
                           metrics, status));
    return LEGEND_OK;
    });
}

int64_t legend_rank_edges_static_max_triples(int32_t dim) {
    if (dim < 1 || dim > max_dim_supported()) return 0;
    const int64_t per_row = (int64_t)rank_dim_padded(dim) * 4 + 8;
    int64_t rows = (int64_t)(kStaticScratchBytes - 3 * 256) / per_row;
    return rows / 64 * 64;
}

int legend_read_embeddings(legend_ctx* c, int32_t table, const int64_t* ids, int64_t m, float* out) {
    return guarded("legend_read_embeddings", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (table < 0 || table > 3) return fail(LEGEND_E_INVAL, "unknown table %d", table);
    if (m < 0) return fail(LEGEND_E_INVAL, "m < 0");
    if (m == 0) return LEGEND_OK;
    if (!out) return fail(LEGEND_E_INVAL, "out must not be NULL");
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->copy));
    HIP_TRY(c, hipStreamSynchronize(c->copy_out));
    for (int s = 0; s < c->nslots; ++s) { c->slot_pending[s] = 0; c->slot_draining[s] = 0; }
    if (c->part_tables_dirty) {
        rc = upload_part_tables(c);
        if (rc) return rc;
    }
    const int d = c->d;
    const size_t rowb = (size_t)d * sizeof(float);
    if (table >= LEGEND_TABLE_REL_EMB) {
        const float* base = table == LEGEND_TABLE_REL_EMB ? c->E_rel : c->S_rel;
        if (!ids) {
            if (m > c->nrel_rows) return fail(LEGEND_E_RANGE, "m exceeds the relation table");
            HIP_TRY(c, hipMemcpy(out, base, (size_t)m * rowb, hipMemcpyDeviceToHost));
            return LEGEND_OK;
        }
        std::vector<float> all((size_t)c->nrel_rows * d);
        HIP_TRY(c, hipMemcpy(all.data(), base, all.size() * sizeof(float), hipMemcpyDeviceToHost));
        for (int64_t k = 0; k < m; ++k) {
            if (ids[k] < 0 || ids[k] >= c->nrel_rows) return fail(LEGEND_E_RANGE, "relation id %lld out of range", (long long)ids[k]);
            std::memcpy(out + k * d, all.data() + ids[k] * d, rowb);
        }
        return LEGEND_OK;
    }
    const size_t off = table == LEGEND_TABLE_NODE_STATE ? (size_t)c->Rp * d : 0;
    if (!ids) {
        if (m > c->V) return fail(LEGEND_E_RANGE, "m exceeds num_nodes");
        for (int p = 0; p < c->n; ++p) {
            int64_t lo = (int64_t)p * c->Rp;
            if (lo >= m) break;
            int64_t rows = std::min<int64_t>(c->Rp, m - lo);
            int sl = c->part_slot[p];
            if (sl >= 0) HIP_TRY(c, hipMemcpy(out + lo * d, c->slot_mem[sl] + off, (size_t)rows * rowb, hipMemcpyDeviceToHost));
            else std::memcpy(out + lo * d, c->host_part[p] + off, (size_t)rows * rowb);
        }
        return LEGEND_OK;
    }
    for (int64_t k = 0; k < m; ++k)
        if (ids[k] < 0 || ids[k] >= c->V) return fail(LEGEND_E_RANGE, "node id %lld out of range", (long long)ids[k]);
    const size_t b_ids = (size_t)m * sizeof(int64_t), b_out = (size_t)m * rowb;
    rc = ensure_io(c, b_ids + b_out + 64);
    if (rc) return rc;
    int64_t* d_ids = reinterpret_cast<int64_t*>(c->io_dev);
    float* d_out = reinterpret_cast<float*>(static_cast<char*>(c->io_dev) + b_ids);
    uint32_t* flag = c->ws.counters + 1;
    HIP_TRY(c, hipMemsetAsync(flag, 0, sizeof(uint32_t), c->compute));
    HIP_TRY(c, hipMemcpyAsync(d_ids, ids, b_ids, hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, launch_gather_rows(c->compute, d_ids, m, table == LEGEND_TABLE_NODE_EMB ? c->d_part_emb : c->d_part_state,
                                  (int32_t)c->Rp, c->V, d, d_out, flag));
    HIP_TRY(c, hipMemcpyAsync(out, d_out, b_out, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    for (int64_t k = 0; k < m; ++k) {
        int p = (int)(ids[k] / c->Rp);
        if (c->part_slot[p] < 0) std::memcpy(out + k * d, c->host_part[p] + off + (ids[k] % c->Rp) * d, rowb);
    }
    return LEGEND_OK;
    });
}

int legend_profile_enable(legend_ctx* c, uint32_t mask) {
    return guarded("legend_profile_enable", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    c->prof_mask = mask & ((1u << KC_COUNT) - 1u);
    return LEGEND_OK;
    });
}

int legend_profile_read(legend_ctx* c, double* ms, int64_t* launches, int32_t capacity) {
    return guarded("legend_profile_read", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!ms || !launches || capacity < KC_COUNT) return fail(LEGEND_E_INVAL, "need capacity >= %d", (int)KC_COUNT);
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    rc = prof_collect(c);
    if (rc) return rc;
    for (int k = 0; k < KC_COUNT; ++k) {
        ms[k] = c->prof_ms[k];
        launches[k] = c->prof_launches[k];
        c->prof_ms[k] = 0.0;
        c->prof_launches[k] = 0;
    }
    return LEGEND_OK;
    });
}

int legend_batch_shape_of(legend_ctx* c, legend_batch_shape* out) {
    return guarded("legend_batch_shape_of", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!out) return fail(LEGEND_E_INVAL, "NULL output");
    out->occurrences = c->gmax.n_occ;
    out->neg_rows = (int64_t)c->gmax.sides * c->gmax.nchunks * c->gmax.T * c->gmax.N;
    out->workspace_bytes = c->gmax.n_occ * (int64_t)(c->d * 4 + 24);
    out->key_bits = c->key_bits;
    out->row_tiles = c->gmax.T;
    return LEGEND_OK;
    });
}

int legend_unique_rows_read(legend_ctx* c, int64_t* unique_rows, int64_t* batches) {
    return guarded("legend_unique_rows_read", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!unique_rows || !batches) return fail(LEGEND_E_INVAL, "NULL output");
    unsigned long long u = 0;
    HIP_TRY(c, hipMemcpyAsync(&u, c->ws.uniq_total, sizeof u, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipMemsetAsync(c->ws.uniq_total, 0, sizeof u, c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    *unique_rows = (int64_t)u;
    *batches = c->batches_done;
    c->batches_done = 0;
    return LEGEND_OK;
    });
}

int legend_fallback_chunks_read(legend_ctx* c, int64_t* chunks) {
    return guarded("legend_fallback_chunks_read", [&]() -> int {
    int rc = check_ctx(c);
    if (rc) return rc;
    if (!chunks) return fail(LEGEND_E_INVAL, "NULL output");
    unsigned long long u = 0;
    HIP_TRY(c, hipMemcpyAsync(&u, c->ws.redo_total, sizeof u, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipMemsetAsync(c->ws.redo_total, 0, sizeof u, c->compute));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    *chunks = (int64_t)u;
    return LEGEND_OK;
    });
}

}  // extern "C"
