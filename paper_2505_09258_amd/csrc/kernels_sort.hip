// The index side of a batch: sort keys of the gradient rows (with the sampled negative ids), a stable
// LSD radix sort of (key, occurrence index) pairs and the segment heads of the sorted keys.  This is
// what makes the deterministic update mode deterministic: equal keys keep their occurrence order, so
// the gradient rows of one table row are always summed in the same order (paper Sec. 2.1 stages 2 and
// 6; the sorting itself is this library's design, the paper does not describe its update kernel).
// Large batches: many short kernels of small workgroups (a histogram, a three-kernel scan and a scatter
// per 8-bit digit), which slip in between the workgroups of the previous batch's kernels with little
// harm.  (A version with a third of the launches -- 8192-key tiles, every scatter workgroup deriving its
// offsets from the whole matrix of tile counts, no scan kernels -- needed less kernel time alone, 133 against
// 180 us per c2 batch, and made the step slower, 1.06 against 1.00 ms: its 512-thread workgroups hold a compute
// unit for 25 us each, and a batch-kernel workgroup needs the unit whole.)  A batch of at most
// kSmallSortMax gradient rows is sorted, cut into segments and planned by one workgroup in one launch.
#include "legend_internal.h"
#include "device_utils.h"
#include "index_side.h"

namespace legend {

// One thread per occurrence (gradient row) of the batch: its sort key, and for negative rows the sampled id.
__global__ void __launch_bounds__(256)
k_prepare(BatchGeom g, BucketParams bp, int32_t* __restrict__ neg_ids, uint32_t* __restrict__ keys) {
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o < g.n_occ) keys[o] = occurrence_key(g, bp, o, neg_ids);
}

hipError_t launch_prepare(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    if (g.n_occ <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((g.n_occ + 255) / 256);
    hipLaunchKernelGGL(k_prepare, dim3(blocks), dim3(256), 0, st, g, bp, ws.neg_ids, ws.keys[0]);
    return hipGetLastError();
}

constexpr int kSortThreads = 256;
constexpr int kSortItems = 8;
constexpr int kSortTile = kSortThreads * kSortItems;   // keys per block
constexpr int kRadix = 256;

// ------------------------------------------------------------------------------------------
// generic exclusive scan of uint32 (three kernels), n <= kSortTile * kSortTile
// MODE 0: value = in[i].  MODE 1: value = head flag of sorted keys in[] (in[i] != in[i-1]).
// ------------------------------------------------------------------------------------------
template <int MODE>
__device__ inline uint32_t scan_value(const uint32_t* __restrict__ in, int64_t i) {
    if (MODE == 0) return in[i];
    return (i == 0 || in[i] != in[i - 1]) ? 1u : 0u;
}

template <int MODE>
__global__ void __launch_bounds__(kSortThreads)
k_scan_reduce(const uint32_t* __restrict__ in, int64_t n, uint32_t* __restrict__ block_sums) {
    __shared__ uint32_t wsum[kSortThreads / kWave];
    int64_t base = (int64_t)blockIdx.x * kSortTile + (int64_t)threadIdx.x * kSortItems;
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        int64_t i = base + k;
        if (i < n) s += scan_value<MODE>(in, i);
    }
    for (int off = kWave / 2; off > 0; off >>= 1) s += __shfl_down(s, off, kWave);
    if (lane_id() == 0) wsum[threadIdx.x / kWave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int w = 0; w < kSortThreads / kWave; ++w) t += wsum[w];
        block_sums[blockIdx.x] = t;
    }
}

// exclusive scan of the block sums in place by one block; total goes to block_sums[nb]
__global__ void __launch_bounds__(kSortThreads)
k_scan_blocksums(uint32_t* __restrict__ block_sums, int nb) {
    __shared__ uint32_t wsum[kSortThreads / kWave];
    __shared__ uint32_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int base = 0; base < nb; base += kSortThreads) {
        int i = base + threadIdx.x;
        uint32_t v = i < nb ? block_sums[i] : 0u;
        uint32_t incl = v;
        for (int off = 1; off < kWave; off <<= 1) {
            uint32_t t = __shfl_up(incl, off, kWave);
            if (lane_id() >= off) incl += t;
        }
        if (lane_id() == kWave - 1) wsum[threadIdx.x / kWave] = incl;
        __syncthreads();
        uint32_t woff = 0;
        for (int w = 0; w < (int)(threadIdx.x / kWave); ++w) woff += wsum[w];
        uint32_t carry = carry_s;
        if (i < nb) block_sums[i] = carry + woff + incl - v;
        __syncthreads();
        if (threadIdx.x == kSortThreads - 1) carry_s = carry + woff + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) block_sums[nb] = carry_s;
}

// MODE 0: out[i] = exclusive prefix.  MODE 1: for head elements write uniq_keys / seg_start.
template <int MODE>
__global__ void __launch_bounds__(kSortThreads)
k_scan_apply(const uint32_t* in, int64_t n, const uint32_t* __restrict__ block_sums,
             uint32_t* out, uint32_t* __restrict__ seg_start, uint32_t* __restrict__ counters,
             unsigned long long* __restrict__ uniq_total, int nb) {
    __shared__ uint32_t wsum[kSortThreads / kWave];
    int64_t base = (int64_t)blockIdx.x * kSortTile + (int64_t)threadIdx.x * kSortItems;
    uint32_t v[kSortItems];
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        int64_t i = base + k;
        v[k] = i < n ? scan_value<MODE>(in, i) : 0u;
        s += v[k];
    }
    uint32_t incl = s;
    for (int off = 1; off < kWave; off <<= 1) {
        uint32_t t = __shfl_up(incl, off, kWave);
        if (lane_id() >= off) incl += t;
    }
    if (lane_id() == kWave - 1) wsum[threadIdx.x / kWave] = incl;
    __syncthreads();
    uint32_t run = block_sums[blockIdx.x] + incl - s;
    for (int w = 0; w < (int)(threadIdx.x / kWave); ++w) run += wsum[w];
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        int64_t i = base + k;
        if (i < n) {
            if (MODE == 0) {
                out[i] = run;
            } else if (v[k]) {
                out[run] = in[i];                 // unique key
                seg_start[run] = (uint32_t)i;     // first sorted position of its segment
            }
        }
        run += v[k];
    }
    if (MODE == 1 && blockIdx.x == 0 && threadIdx.x == 0) {
        uint32_t total = block_sums[nb];
        seg_start[total] = (uint32_t)n;
        counters[0] = total;
        counters[2] = 0;                      // the update kernels count long rows and their units here
        counters[3] = 0;
        *uniq_total += total;
    }
}

static hipError_t scan_launch(hipStream_t st, int mode, const uint32_t* in, int64_t n, uint32_t* tmp,
                              uint32_t* out, uint32_t* seg_start, uint32_t* counters,
                              unsigned long long* uniq_total) {
    int nb = (int)((n + kSortTile - 1) / kSortTile);
    if (nb > kSortTile) return hipErrorInvalidValue;
    if (mode == 0) {
        hipLaunchKernelGGL(k_scan_reduce<0>, dim3(nb), dim3(kSortThreads), 0, st, in, n, tmp);
        hipLaunchKernelGGL(k_scan_blocksums, dim3(1), dim3(kSortThreads), 0, st, tmp, nb);
        hipLaunchKernelGGL(k_scan_apply<0>, dim3(nb), dim3(kSortThreads), 0, st, in, n, tmp, out, seg_start,
                           counters, uniq_total, nb);
    } else {
        hipLaunchKernelGGL(k_scan_reduce<1>, dim3(nb), dim3(kSortThreads), 0, st, in, n, tmp);
        hipLaunchKernelGGL(k_scan_blocksums, dim3(1), dim3(kSortThreads), 0, st, tmp, nb);
        hipLaunchKernelGGL(k_scan_apply<1>, dim3(nb), dim3(kSortThreads), 0, st, in, n, tmp, out, seg_start,
                           counters, uniq_total, nb);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// radix sort pass
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kSortThreads)
k_radix_hist(const uint32_t* __restrict__ keys, int64_t n, int shift, uint32_t* __restrict__ ghist, int nblk) {
    __shared__ uint32_t h[kRadix];
    h[threadIdx.x] = 0;
    __syncthreads();
    int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        int64_t i = base + k * kSortThreads + threadIdx.x;
        if (i < n) atomicAdd(&h[(keys[i] >> shift) & (kRadix - 1)], 1u);
    }
    __syncthreads();
    ghist[(int64_t)threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];
}

// Stable scatter.  Wave w of a block owns 512 consecutive keys and walks them in 8
// rounds of 64; the rank of a key among equal digits is (equal digits in earlier
// waves) + (in earlier rounds of this wave) + (in lower lanes of this round).
__global__ void __launch_bounds__(kSortThreads)
k_radix_scatter(const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ vals_in,
                uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out, int64_t n, int shift,
                const uint32_t* __restrict__ goff, int nblk) {
    constexpr int kWaves = kSortThreads / kWave;
    __shared__ uint32_t cnt[kWaves][kRadix];
    __shared__ uint32_t pos0[kWaves][kRadix];
    for (int i = threadIdx.x; i < kWaves * kRadix; i += kSortThreads) (&cnt[0][0])[i] = 0;
    __syncthreads();
    const int w = threadIdx.x / kWave;
    const int lane = lane_id();
    volatile uint32_t* mycnt = cnt[w];
    const int64_t wbase = (int64_t)blockIdx.x * kSortTile + (int64_t)w * (kWave * kSortItems);
    uint32_t key[kSortItems];
    uint32_t rank[kSortItems];
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        int64_t i = wbase + r * kWave + lane;
        bool valid = i < n;
        key[r] = valid ? keys_in[i] : 0u;
        uint32_t digit = (key[r] >> shift) & (kRadix - 1);
        unsigned long long mask = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            bool bit = (digit >> b) & 1u;
            unsigned long long m = __ballot(bit);
            mask &= bit ? m : ~m;
        }
        unsigned long long lower = mask & ((1ull << lane) - 1ull);
        uint32_t prefix = 0;
        if (valid) prefix = mycnt[digit];
        if (valid && lower == 0ull) mycnt[digit] = prefix + (uint32_t)__popcll(mask);
        rank[r] = prefix + (uint32_t)__popcll(lower);
    }
    __syncthreads();
    {
        int d = threadIdx.x;
        uint32_t run = goff[(int64_t)d * nblk + blockIdx.x];
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) {
            pos0[ww][d] = run;
            run += cnt[ww][d];
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        int64_t i = wbase + r * kWave + lane;
        if (i < n) {
            uint32_t digit = (key[r] >> shift) & (kRadix - 1);
            uint32_t p = pos0[w][digit] + rank[r];
            keys_out[p] = key[r];
            vals_out[p] = vals_in ? vals_in[i] : (uint32_t)i;
        }
    }
}

static hipError_t launch_sort(hipStream_t st, int64_t n, int key_bits, const Workspace& ws, int* out_buf) {
    *out_buf = 0;
    if (n <= 0) return hipSuccess;
    int passes = (key_bits + 7) / 8;
    if (passes < 1) passes = 1;
    int nblk = (int)((n + kSortTile - 1) / kSortTile);
    int cur = 0;
    for (int p = 0; p < passes; ++p) {
        int shift = 8 * p;
        hipLaunchKernelGGL(k_radix_hist, dim3(nblk), dim3(kSortThreads), 0, st, ws.keys[cur], n, shift, ws.ghist, nblk);
        hipError_t e = scan_launch(st, 0, ws.ghist, (int64_t)kRadix * nblk, ws.scan_tmp, ws.ghist, nullptr, nullptr, nullptr);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k_radix_scatter, dim3(nblk), dim3(kSortThreads), 0, st, ws.keys[cur],
                           p == 0 ? (const uint32_t*)nullptr : ws.vals[cur], ws.keys[cur ^ 1], ws.vals[cur ^ 1], n,
                           shift, ws.ghist, nblk);
        cur ^= 1;
    }
    *out_buf = cur;
    return hipGetLastError();
}

static hipError_t launch_segments(hipStream_t st, int64_t n, const uint32_t* sorted_keys, const Workspace& ws) {
    if (n <= 0) return hipSuccess;
    return scan_launch(st, 1, sorted_keys, n, ws.scan_tmp, ws.uniq_keys, ws.seg_start, ws.counters, ws.uniq_total);
}

// ------------------------------------------------------------------------------------------
// Small batches (n <= kSmallSortMax): one workgroup sorts the pairs in LDS, emits the segment
// heads and (deterministic mode) lists the rows with many gradient rows and their units, so a
// latency-bound tiny batch pays one launch instead of some twenty.  (Making the keys in this kernel
// as well was tried: one workgroup walking a few thousand occurrences, each with its 64-bit index
// arithmetic and hashes, took longer than the launch it saved: 89 against 54 us per c1 batch.)
// Same stable ranking as the multi-block scatter: wave w of the sixteen owns a contiguous share of the keys.
// ------------------------------------------------------------------------------------------

constexpr int kSmallThreads = 1024;
static_assert(kSmallThreads >= kRadix && kSmallSortMax % kSmallThreads == 0, "small sort geometry");

__global__ void __launch_bounds__(kSmallThreads)
k_small_sort_segments(const uint32_t* __restrict__ keys_in, int n, int passes, uint32_t* __restrict__ vals_out,
                      uint32_t* __restrict__ uniq_keys, uint32_t* __restrict__ seg_start,
                      uint32_t* __restrict__ counters, unsigned long long* __restrict__ uniq_total,
                      uint32_t* __restrict__ long_list, uint32_t* __restrict__ unit_start, int plan_long) {
    constexpr int kWaves = kSmallThreads / kWave;
    extern __shared__ uint32_t sm[];
    auto kb = [&](int b) { return sm + b * kSmallSortMax; };                     // key buffers 0 / 1
    auto vb = [&](int b) { return sm + (2 + b) * kSmallSortMax; };               // value buffers 0 / 1
    uint32_t* cnt = sm + 4 * kSmallSortMax;            // [kWaves][256]
    uint32_t* pos0 = cnt + kWaves * kRadix;            // [kWaves][256]
    uint32_t* wsum = pos0 + kWaves * kRadix;           // [kWaves] + carry
    const int tid = threadIdx.x, w = tid / kWave, lane = lane_id();
    for (int i = tid; i < n; i += kSmallThreads) { kb(0)[i] = keys_in[i]; vb(0)[i] = (uint32_t)i; }
    __syncthreads();
    const int per_wave = (n + kWaves - 1) / kWaves;
    const int lo = min(n, w * per_wave), hi = min(n, lo + per_wave);
    int cur = 0;
    for (int p = 0; p < passes; ++p) {
        const int shift = 8 * p;
        for (int i = tid; i < kWaves * kRadix; i += kSmallThreads) cnt[i] = 0;
        __syncthreads();
        volatile uint32_t* mycnt = cnt + w * kRadix;
        // pass 1 over the wave's keys: rank among equal digits inside the wave (kept in pos0's place later)
        for (int base = lo; base < hi; base += kWave) {
            const int i = base + lane;
            const bool valid = i < hi;
            const uint32_t key = valid ? kb(cur)[i] : 0u;
            const uint32_t digit = (key >> shift) & (kRadix - 1);
            unsigned long long mask = __ballot(valid);
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const bool bit = (digit >> b) & 1u;
                const unsigned long long m = __ballot(bit);
                mask &= bit ? m : ~m;
            }
            const unsigned long long lower = mask & ((1ull << lane) - 1ull);
            uint32_t prefix = 0;
            if (valid) prefix = mycnt[digit];
            if (valid && lower == 0ull) mycnt[digit] = prefix + (uint32_t)__popcll(mask);
            if (valid) vb(cur ^ 1)[i] = prefix + (uint32_t)__popcll(lower);   // rank, parked in the spare buffer
        }
        __syncthreads();
        // exclusive scan over digits of the per-digit totals (the first kRadix threads, one digit each), then
        // per-wave starting positions
        {
            const int d = tid;
            uint32_t tot = 0;
            if (d < kRadix) {
#pragma unroll
                for (int ww = 0; ww < kWaves; ++ww) tot += cnt[ww * kRadix + d];
            }
            uint32_t incl = tot;
            for (int off = 1; off < kWave; off <<= 1) {
                const uint32_t t = __shfl_up(incl, off, kWave);
                if (lane >= off) incl += t;
            }
            if (d < kRadix && lane == kWave - 1) wsum[w] = incl;
            __syncthreads();
            if (d < kRadix) {
                uint32_t run = incl - tot;
                for (int ww = 0; ww < w; ++ww) run += wsum[ww];
#pragma unroll
                for (int ww = 0; ww < kWaves; ++ww) {
                    pos0[ww * kRadix + d] = run;
                    run += cnt[ww * kRadix + d];
                }
            }
        }
        __syncthreads();
        // scatter: ranks were parked in vbuf[cur^1]; move pairs through registers to avoid overwriting them
        uint32_t mk[kSmallSortMax / kSmallThreads], mv[kSmallSortMax / kSmallThreads], mp[kSmallSortMax / kSmallThreads];
#pragma unroll
        for (int r = 0; r < kSmallSortMax / kSmallThreads; ++r) {
            const int i = tid + r * kSmallThreads;
            if (i < n) {
                const int ww = min(kWaves - 1, i / per_wave);
                mk[r] = kb(cur)[i];
                mv[r] = vb(cur)[i];
                mp[r] = pos0[ww * kRadix + ((mk[r] >> shift) & (kRadix - 1))] + vb(cur ^ 1)[i];
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kSmallSortMax / kSmallThreads; ++r) {
            const int i = tid + r * kSmallThreads;
            if (i < n) { kb(cur ^ 1)[mp[r]] = mk[r]; vb(cur ^ 1)[mp[r]] = mv[r]; }
        }
        __syncthreads();
        cur ^= 1;
    }
    // sorted values out; segment heads by a block scan of the head flags
    for (int i = tid; i < n; i += kSmallThreads) vals_out[i] = vb(cur)[i];
    if (tid == 0) wsum[kWaves] = 0;
    __syncthreads();
    for (int base = 0; base < n; base += kSmallThreads) {
        const int i = base + tid;
        const uint32_t key = i < n ? kb(cur)[i] : 0u;
        const uint32_t flag = (i < n && (i == 0 || key != kb(cur)[i - 1])) ? 1u : 0u;
        uint32_t incl = flag;
        for (int off = 1; off < kWave; off <<= 1) {
            const uint32_t t = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += t;
        }
        if (lane == kWave - 1) wsum[w] = incl;
        __syncthreads();
        uint32_t run = wsum[kWaves] + incl - flag;
        for (int ww = 0; ww < w; ++ww) run += wsum[ww];
        if (flag) { uniq_keys[run] = key; seg_start[run] = (uint32_t)i; }
        __syncthreads();
        if (tid == kSmallThreads - 1) wsum[kWaves] = run + flag;
        __syncthreads();
    }
    const uint32_t total = wsum[kWaves];
    if (tid == 0) {
        seg_start[total] = (uint32_t)n;
        counters[0] = total;
        *uniq_total += total;
        wsum[kWaves + 1] = 0;                 // long rows
        wsum[kWaves + 2] = 0;                 // their units
    }
    __threadfence_block();                    // segment bounds written above are read by other lanes below
    __syncthreads();
    uint32_t n_long = 0, units = 0;
    if (plan_long) {
        // table rows with many gradient rows, in no particular order, then the exclusive prefix of
        // their unit counts
        for (uint32_t u = tid; u < total; u += kSmallThreads)
            if (seg_start[u + 1] - seg_start[u] > (uint32_t)kLongLen) long_list[atomicAdd(&wsum[kWaves + 1], 1u)] = u;
        __threadfence_block();
        __syncthreads();
        n_long = wsum[kWaves + 1];
        for (uint32_t base = 0; base < n_long; base += kSmallThreads) {
            const uint32_t r = base + tid;
            uint32_t v = 0;
            if (r < n_long) {
                const uint32_t u = long_list[r];
                v = (seg_start[u + 1] - seg_start[u] + kUnit - 1) / kUnit;
            }
            uint32_t incl = v;
            for (int off = 1; off < kWave; off <<= 1) {
                const uint32_t t = __shfl_up(incl, off, kWave);
                if (lane >= off) incl += t;
            }
            if (lane == kWave - 1) wsum[w] = incl;
            __syncthreads();
            uint32_t woff = 0;
            for (int ww = 0; ww < w; ++ww) woff += wsum[ww];
            const uint32_t carry = wsum[kWaves + 2];
            if (r < n_long) unit_start[r] = carry + woff + incl - v;
            __syncthreads();
            if (tid == kSmallThreads - 1) wsum[kWaves + 2] = carry + woff + incl;
            __syncthreads();
        }
        units = wsum[kWaves + 2];
    }
    if (tid == 0) {
        if (plan_long) unit_start[n_long] = units;
        counters[2] = n_long;
        counters[3] = units;
    }
}

hipError_t launch_sort_and_segments(hipStream_t st, const BatchGeom& g, const BucketParams& bp, int key_bits,
                                    const Workspace& ws, int* out_buf, bool plan_long) {
    *out_buf = 0;
    const int64_t n = g.n_occ;
    if (n <= 0) return hipSuccess;
    int passes = (key_bits + 7) / 8;
    if (passes < 1) passes = 1;
    if (n <= kSmallSortMax) {
        const size_t lds = (4 * (size_t)kSmallSortMax + 2 * (kSmallThreads / kWave) * kRadix + (kSmallThreads / kWave) + 8) * sizeof(uint32_t);
        static PerDeviceFlag attr_set;
        if (attr_set.pending()) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_small_sort_segments),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set.set();
        }
        hipLaunchKernelGGL(k_small_sort_segments, dim3(1), dim3(kSmallThreads), lds, st, ws.keys[0], (int)n, passes,
                           ws.vals[1], ws.uniq_keys, ws.seg_start, ws.counters, ws.uniq_total, ws.long_list,
                           ws.unit_start, plan_long ? 1 : 0);
        *out_buf = 1;
        return hipGetLastError();
    }
    hipError_t e = launch_sort(st, n, key_bits, ws, out_buf);
    if (e != hipSuccess) return e;
    return launch_segments(st, n, ws.keys[*out_buf], ws);
}

}  // namespace legend
