// Embedding update (paper Sec. 2.1 stage 6, Sec. 3 step 5) and the read-side kernels.
//
// Deterministic mode: the sorted occurrence list groups the staged gradient rows by
// table row; each group is summed in occurrence order in fp64, rounded once to fp32,
// and the textbook Adagrad rule is applied in fp32 (the paper names Adagrad, Sec. 2.1,
// without printing it):  S <- S + G*G ;  theta <- theta - lr * G / (sqrt(S) + eps).
#include "legend_internal.h"
#include "device_utils.h"

namespace legend {

struct UpdateTables {
    float* E[3];
    float* S[3];
    uint32_t key_base[3];   // first key of table slot 0 (partition i), 1 (partition j), 2 (relations)
};

__device__ inline void adagrad_elem(float g, float& theta, float& state, float lr, float eps) {
#pragma clang fp contract(off)
    float g2 = g * g;
    float s = state + g2;
    float num = lr * g;
    float den = sqrtf(s) + eps;
    float step = num / den;
    state = s;
    theta = theta - step;
}

__device__ inline int table_of_key(const UpdateTables& tb, uint32_t key) {
    return key >= tb.key_base[2] ? 2 : (key >= tb.key_base[1] && tb.key_base[1] > 0 ? 1 : 0);
}

// Sum of gradient rows sorted_vals[lo..hi) (columns c0..c0+3) in that order, in fp64.
__device__ inline void sum_rows(const float* __restrict__ grad, const uint32_t* __restrict__ sorted_vals,
                                uint32_t lo, uint32_t hi, int d, int c0, bool vec4, double acc[4]) {
    uint32_t p = lo;
    if (vec4) {
        for (; p + 4 <= hi; p += 4) {           // four independent loads in flight, added in order
            const uint32_t o0 = sorted_vals[p], o1 = sorted_vals[p + 1], o2 = sorted_vals[p + 2], o3 = sorted_vals[p + 3];
            const float4 v0 = *reinterpret_cast<const float4*>(grad + (int64_t)o0 * d + c0);
            const float4 v1 = *reinterpret_cast<const float4*>(grad + (int64_t)o1 * d + c0);
            const float4 v2 = *reinterpret_cast<const float4*>(grad + (int64_t)o2 * d + c0);
            const float4 v3 = *reinterpret_cast<const float4*>(grad + (int64_t)o3 * d + c0);
            acc[0] += (double)v0.x; acc[1] += (double)v0.y; acc[2] += (double)v0.z; acc[3] += (double)v0.w;
            acc[0] += (double)v1.x; acc[1] += (double)v1.y; acc[2] += (double)v1.z; acc[3] += (double)v1.w;
            acc[0] += (double)v2.x; acc[1] += (double)v2.y; acc[2] += (double)v2.z; acc[3] += (double)v2.w;
            acc[0] += (double)v3.x; acc[1] += (double)v3.y; acc[2] += (double)v3.z; acc[3] += (double)v3.w;
        }
        // one to three rows left (the common case: most table rows get one or two gradient rows):
        // their loads go out together as well, the sums stay in order
        const uint32_t n = hi - p;
        if (n == 1) {
            const float4 v0 = *reinterpret_cast<const float4*>(grad + (int64_t)sorted_vals[p] * d + c0);
            acc[0] += (double)v0.x; acc[1] += (double)v0.y; acc[2] += (double)v0.z; acc[3] += (double)v0.w;
        } else if (n == 2) {
            const uint32_t o0 = sorted_vals[p], o1 = sorted_vals[p + 1];
            const float4 v0 = *reinterpret_cast<const float4*>(grad + (int64_t)o0 * d + c0);
            const float4 v1 = *reinterpret_cast<const float4*>(grad + (int64_t)o1 * d + c0);
            acc[0] += (double)v0.x; acc[1] += (double)v0.y; acc[2] += (double)v0.z; acc[3] += (double)v0.w;
            acc[0] += (double)v1.x; acc[1] += (double)v1.y; acc[2] += (double)v1.z; acc[3] += (double)v1.w;
        } else if (n == 3) {
            const uint32_t o0 = sorted_vals[p], o1 = sorted_vals[p + 1], o2 = sorted_vals[p + 2];
            const float4 v0 = *reinterpret_cast<const float4*>(grad + (int64_t)o0 * d + c0);
            const float4 v1 = *reinterpret_cast<const float4*>(grad + (int64_t)o1 * d + c0);
            const float4 v2 = *reinterpret_cast<const float4*>(grad + (int64_t)o2 * d + c0);
            acc[0] += (double)v0.x; acc[1] += (double)v0.y; acc[2] += (double)v0.z; acc[3] += (double)v0.w;
            acc[0] += (double)v1.x; acc[1] += (double)v1.y; acc[2] += (double)v1.z; acc[3] += (double)v1.w;
            acc[0] += (double)v2.x; acc[1] += (double)v2.y; acc[2] += (double)v2.z; acc[3] += (double)v2.w;
        }
    } else if ((d & 1) == 0) {
        // an even dimension that is no multiple of four (50 and 150 of the paper's dimension sweep): rows are
        // 8-byte aligned, two 64-bit loads per gradient row, four rows in flight, added in order
        const bool second = c0 + 2 < d;
        auto row2 = [&](uint32_t o, float2& a, float2& b) {
            const float* gp = grad + (int64_t)o * d + c0;
            a = *reinterpret_cast<const float2*>(gp);
            b = second ? *reinterpret_cast<const float2*>(gp + 2) : make_float2(0.f, 0.f);
        };
        for (; p + 4 <= hi; p += 4) {
            float2 a0, b0, a1, b1, a2, b2, a3, b3;
            row2(sorted_vals[p], a0, b0);
            row2(sorted_vals[p + 1], a1, b1);
            row2(sorted_vals[p + 2], a2, b2);
            row2(sorted_vals[p + 3], a3, b3);
            acc[0] += (double)a0.x; acc[1] += (double)a0.y; acc[2] += (double)b0.x; acc[3] += (double)b0.y;
            acc[0] += (double)a1.x; acc[1] += (double)a1.y; acc[2] += (double)b1.x; acc[3] += (double)b1.y;
            acc[0] += (double)a2.x; acc[1] += (double)a2.y; acc[2] += (double)b2.x; acc[3] += (double)b2.y;
            acc[0] += (double)a3.x; acc[1] += (double)a3.y; acc[2] += (double)b3.x; acc[3] += (double)b3.y;
        }
        for (; p < hi; ++p) {
            float2 a0, b0;
            row2(sorted_vals[p], a0, b0);
            acc[0] += (double)a0.x; acc[1] += (double)a0.y; acc[2] += (double)b0.x; acc[3] += (double)b0.y;
        }
    } else {
        for (; p < hi; ++p) {
            const float* gp = grad + (int64_t)sorted_vals[p] * d + c0;
            acc[0] += (double)gp[0];
            if (c0 + 1 < d) acc[1] += (double)gp[1];
            if (c0 + 2 < d) acc[2] += (double)gp[2];
            if (c0 + 3 < d) acc[3] += (double)gp[3];
        }
    }
}

__device__ inline void apply_row(const UpdateTables& tb, uint32_t key, const double acc[4], int d, int c0, bool vec4,
                                 float lr, float eps) {
    const int t = table_of_key(tb, key);
    const int64_t row = (int64_t)(key - tb.key_base[t]);
    float* ep = tb.E[t] + row * d + c0;
    float* sp = tb.S[t] + row * d + c0;
    if (vec4) {
        float4 th = *reinterpret_cast<float4*>(ep);
        float4 st = *reinterpret_cast<float4*>(sp);
        adagrad_elem((float)acc[0], th.x, st.x, lr, eps);
        adagrad_elem((float)acc[1], th.y, st.y, lr, eps);
        adagrad_elem((float)acc[2], th.z, st.z, lr, eps);
        adagrad_elem((float)acc[3], th.w, st.w, lr, eps);
        *reinterpret_cast<float4*>(ep) = th;
        *reinterpret_cast<float4*>(sp) = st;
    } else if ((d & 1) == 0) {
        const bool second = c0 + 2 < d;
        float2 ta = *reinterpret_cast<float2*>(ep), sa = *reinterpret_cast<float2*>(sp);
        float2 tb2 = make_float2(0.f, 0.f), sb2 = make_float2(0.f, 0.f);
        if (second) { tb2 = *reinterpret_cast<float2*>(ep + 2); sb2 = *reinterpret_cast<float2*>(sp + 2); }
        adagrad_elem((float)acc[0], ta.x, sa.x, lr, eps);
        adagrad_elem((float)acc[1], ta.y, sa.y, lr, eps);
        *reinterpret_cast<float2*>(ep) = ta;
        *reinterpret_cast<float2*>(sp) = sa;
        if (second) {
            adagrad_elem((float)acc[2], tb2.x, sb2.x, lr, eps);
            adagrad_elem((float)acc[3], tb2.y, sb2.y, lr, eps);
            *reinterpret_cast<float2*>(ep + 2) = tb2;
            *reinterpret_cast<float2*>(sp + 2) = sb2;
        }
    } else {
        for (int j = 0; j < 4 && c0 + j < d; ++j) {
            float th = ep[j], st = sp[j];
            adagrad_elem((float)acc[j], th, st, lr, eps);
            ep[j] = th;
            sp[j] = st;
        }
    }
}

// Table rows with many gradient rows (counters[2] = how many, long_list = which, in no particular
// order: every such row is handled on its own).  Part of the index side of a batch: it depends
// on the segment bounds only.
__global__ void __launch_bounds__(256)
k_long_list(uint32_t* __restrict__ counters, const uint32_t* __restrict__ seg_start, uint32_t* __restrict__ long_list) {
    const uint32_t n_unique = counters[0];
    for (uint32_t u = blockIdx.x * 256 + threadIdx.x; u < n_unique; u += gridDim.x * 256)
        if (seg_start[u + 1] - seg_start[u] > (uint32_t)kLongLen) long_list[atomicAdd(&counters[2], 1u)] = u;
}

// LPR lanes (a float4 each) own one table row: the rows u0, u0 + stride, ... of the batch's unique rows.
// Rows with many gradient rows are left to the kernels below.
template <int LPR>
__device__ inline void update_short_rows(uint32_t u0, uint32_t stride, uint32_t n_unique,
                                         const uint32_t* __restrict__ uniq_keys, const uint32_t* __restrict__ seg_start,
                                         const uint32_t* __restrict__ sorted_vals, const float* __restrict__ grad,
                                         const UpdateTables& tb, int d, float lr, float eps) {
    const int col4 = threadIdx.x % LPR;
    const int c0 = col4 * 4;
    const bool vec4 = (d & 3) == 0;
    for (uint32_t u = u0; u < n_unique; u += stride) {
        const uint32_t lo = seg_start[u], hi = seg_start[u + 1];
        if (hi - lo > (uint32_t)kLongLen) continue;
        if (vec4 && d <= 4 * LPR) {
            // one pass over the row: the table row's loads are issued before the gradient rows are
            // summed, so that the two round trips to memory overlap
            if (c0 < d) {
                const uint32_t key = uniq_keys[u];
                const int t = table_of_key(tb, key);
                const int64_t row = (int64_t)(key - tb.key_base[t]);
                float* ep = tb.E[t] + row * d + c0;
                float* sp = tb.S[t] + row * d + c0;
                float4 th = *reinterpret_cast<const float4*>(ep);
                float4 st = *reinterpret_cast<const float4*>(sp);
                double acc[4] = {0.0, 0.0, 0.0, 0.0};
                sum_rows(grad, sorted_vals, lo, hi, d, c0, true, acc);
                adagrad_elem((float)acc[0], th.x, st.x, lr, eps);
                adagrad_elem((float)acc[1], th.y, st.y, lr, eps);
                adagrad_elem((float)acc[2], th.z, st.z, lr, eps);
                adagrad_elem((float)acc[3], th.w, st.w, lr, eps);
                *reinterpret_cast<float4*>(ep) = th;
                *reinterpret_cast<float4*>(sp) = st;
            }
            continue;
        }
        for (int cc = c0; cc < d; cc += 4 * LPR) {     // rows wider than 4*LPR floats take several passes
            double acc[4] = {0.0, 0.0, 0.0, 0.0};
            sum_rows(grad, sorted_vals, lo, hi, d, cc, vec4, acc);
            apply_row(tb, uniq_keys[u], acc, d, cc, vec4, lr, eps);
        }
    }
}

template <int LPR>
__global__ void __launch_bounds__(256)
k_update(const uint32_t* __restrict__ counters, const uint32_t* __restrict__ uniq_keys,
         const uint32_t* __restrict__ seg_start, const uint32_t* __restrict__ sorted_vals,
         const float* __restrict__ grad, UpdateTables tb, int d, float lr, float eps) {
    constexpr int groups_per_block = 256 / LPR;
    update_short_rows<LPR>(blockIdx.x * groups_per_block + threadIdx.x / LPR, gridDim.x * groups_per_block, counters[0],
                           uniq_keys, seg_start, sorted_vals, grad, tb, d, lr, eps);
}

// Units of the two-level path: long row r owns ceil(len / kUnit) consecutive units;
// unit_start = exclusive prefix of those counts (one block, sequential over blocks of 256).
__global__ void __launch_bounds__(256)
k_long_plan(uint32_t* __restrict__ counters, const uint32_t* __restrict__ long_list,
            const uint32_t* __restrict__ seg_start, uint32_t* __restrict__ unit_start) {
    __shared__ uint32_t wsum[4];
    __shared__ uint32_t carry_s;
    const uint32_t n_long = counters[2];
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (uint32_t base = 0; base < n_long; base += 256) {
        const uint32_t r = base + threadIdx.x;
        uint32_t v = 0;
        if (r < n_long) {
            const uint32_t u = long_list[r];
            v = (seg_start[u + 1] - seg_start[u] + kUnit - 1) / kUnit;
        }
        uint32_t incl = v;
        for (int off = 1; off < kWave; off <<= 1) {
            uint32_t t = __shfl_up(incl, off, kWave);
            if (lane_id() >= off) incl += t;
        }
        if (lane_id() == kWave - 1) wsum[threadIdx.x / kWave] = incl;
        __syncthreads();
        uint32_t woff = 0;
        for (int w = 0; w < (int)(threadIdx.x / kWave); ++w) woff += wsum[w];
        const uint32_t carry = carry_s;
        if (r < n_long) unit_start[r] = carry + woff + incl - v;
        __syncthreads();
        if (threadIdx.x == 255) carry_s = carry + woff + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        unit_start[n_long] = carry_s;
        counters[3] = carry_s;
    }
}

// One block per unit: the block's groups sum kUnit / GROUPS consecutive gradient rows each, the partial
// sums are added in group order by the lanes of group 0, which get the unit's fp64 sum of columns cc..cc+3.
template <int LPR>
__device__ inline void unit_sum(uint32_t lo_unit, uint32_t seg_hi, const uint32_t* __restrict__ sorted_vals,
                                const float* __restrict__ grad, int d, int cbase, bool vec4, double* psum, double tot[4]) {
    constexpr int GROUPS = 256 / LPR;
    constexpr int PER_GROUP = kUnit / GROUPS;
    const int gl = threadIdx.x / LPR;
    const int col4 = threadIdx.x % LPR;
    const int cc = cbase + col4 * 4;
    const uint32_t lo = lo_unit + gl * PER_GROUP;
    const uint32_t hi = min(seg_hi, lo + PER_GROUP);
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    if (cc < d && lo < hi) sum_rows(grad, sorted_vals, lo, hi, d, cc, vec4, acc);
#pragma unroll
    for (int j = 0; j < 4; ++j) psum[(gl * LPR + col4) * 4 + j] = acc[j];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) tot[j] = 0.0;
    if (gl == 0 && cc < d) {
        for (int gq = 0; gq < GROUPS; ++gq)
#pragma unroll
            for (int j = 0; j < 4; ++j) tot[j] += psum[(gq * LPR + col4) * 4 + j];
    }
    __syncthreads();
}

template <int LPR>
__global__ void __launch_bounds__(256)
k_long_partial(const uint32_t* __restrict__ counters, const uint32_t* __restrict__ long_list,
               const uint32_t* __restrict__ unit_start, const uint32_t* __restrict__ seg_start,
               const uint32_t* __restrict__ sorted_vals, const float* __restrict__ grad, int d,
               double* __restrict__ partial) {
    extern __shared__ double psum[];          // [GROUPS][4 * LPR]
    const int gl = threadIdx.x / LPR;
    const int col4 = threadIdx.x % LPR;
    const bool vec4 = (d & 3) == 0;
    const uint32_t n_long = counters[2], n_units = counters[3];
    for (uint32_t unit = blockIdx.x; unit < n_units; unit += gridDim.x) {
        uint32_t a = 0, b = n_long;           // last r with unit_start[r] <= unit
        while (b - a > 1) {
            uint32_t mid = (a + b) >> 1;
            if (unit_start[mid] <= unit) a = mid; else b = mid;
        }
        const uint32_t u = long_list[a];
        const uint32_t seg_lo = seg_start[u], seg_hi = seg_start[u + 1];
        for (int cbase = 0; cbase < d; cbase += 4 * LPR) {     // uniform trip count across the block
            const int cc = cbase + col4 * 4;
            double tot[4];
            unit_sum<LPR>(seg_lo + (unit - unit_start[a]) * kUnit, seg_hi, sorted_vals, grad, d, cbase, vec4, psum, tot);
            if (gl == 0 && cc < d)
                for (int j = 0; j < 4 && cc + j < d; ++j) partial[(int64_t)unit * d + cc + j] = tot[j];
        }
    }
}

// One group per long row: its units' partial rows are added in unit order, then Adagrad.
template <int LPR>
__global__ void __launch_bounds__(256)
k_long_final(const uint32_t* __restrict__ counters, const uint32_t* __restrict__ long_list,
             const uint32_t* __restrict__ unit_start, const uint32_t* __restrict__ uniq_keys,
             const double* __restrict__ partial, UpdateTables tb, int d, float lr, float eps) {
    const int groups_per_block = 256 / LPR;
    const int gl = threadIdx.x / LPR;
    const int col4 = threadIdx.x % LPR;
    const int c0 = col4 * 4;
    const bool vec4 = (d & 3) == 0;
    const uint32_t n_long = counters[2];
    for (uint32_t r = blockIdx.x * groups_per_block + gl; r < n_long; r += gridDim.x * groups_per_block) {
        for (int cc = c0; cc < d; cc += 4 * LPR) {
            double acc[4] = {0.0, 0.0, 0.0, 0.0};
            for (uint32_t unit = unit_start[r]; unit < unit_start[r + 1]; ++unit) {
                const double* pp = partial + (int64_t)unit * d + cc;
                for (int j = 0; j < 4 && cc + j < d; ++j) acc[j] += pp[j];
            }
            apply_row(tb, uniq_keys[long_list[r]], acc, d, cc, vec4, lr, eps);
        }
    }
}

// A batch of at most kSmallSortMax gradient rows is bound by launch latency: one launch does what
// k_loss_reduce, k_update, k_long_partial and k_long_final do, with the same sums in the same order.
//   blocks [0, row_blocks)            the table rows with few gradient rows
//   blocks [row_blocks, gridDim - 1)  one block per table row with many: its units one after the other
//   the last block                    the sum of the workgroups' loss terms
template <int LPR>
__global__ void __launch_bounds__(256)
k_update_small(const uint32_t* __restrict__ counters, const uint32_t* __restrict__ uniq_keys,
               const uint32_t* __restrict__ seg_start, const uint32_t* __restrict__ sorted_vals,
               const uint32_t* __restrict__ long_list, const float* __restrict__ grad, UpdateTables tb, int d, float lr,
               float eps, int row_blocks, const double* __restrict__ loss_partial, int64_t loss_n,
               double* __restrict__ loss_sum) {
    __shared__ double psum[4 * 256];
    constexpr int groups_per_block = 256 / LPR;
    const int b = blockIdx.x;
    if (b < row_blocks) {
        update_short_rows<LPR>(b * groups_per_block + threadIdx.x / LPR, row_blocks * groups_per_block, counters[0],
                               uniq_keys, seg_start, sorted_vals, grad, tb, d, lr, eps);
        return;
    }
    if (b == (int)gridDim.x - 1) {
        double s = 0.0;
        for (int64_t i = threadIdx.x; i < loss_n; i += 256) s += loss_partial[i];
        psum[threadIdx.x] = s;
        __syncthreads();
        for (int off = 128; off > 0; off >>= 1) {
            if ((int)threadIdx.x < off) psum[threadIdx.x] += psum[threadIdx.x + off];
            __syncthreads();
        }
        if (threadIdx.x == 0 && loss_n > 0) *loss_sum += psum[0];
        return;
    }
    const uint32_t r = (uint32_t)(b - row_blocks);
    if (r >= counters[2]) return;                              // uniform
    const uint32_t u = long_list[r];
    const uint32_t seg_lo = seg_start[u], seg_hi = seg_start[u + 1];
    const bool vec4 = (d & 3) == 0;
    const int gl = threadIdx.x / LPR, col4 = threadIdx.x % LPR;
    for (int cbase = 0; cbase < d; cbase += 4 * LPR) {
        const int cc = cbase + col4 * 4;
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        for (uint32_t lo = seg_lo; lo < seg_hi; lo += kUnit) {
            double tot[4];
            unit_sum<LPR>(lo, seg_hi, sorted_vals, grad, d, cbase, vec4, psum, tot);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] += tot[j];
        }
        if (gl == 0 && cc < d) apply_row(tb, uniq_keys[u], acc, d, cc, vec4, lr, eps);
    }
}

template <int LPR>
static hipError_t launch_update_lpr(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws,
                                    const uint32_t* sorted_vals, const UpdateTables& tb, bool long_rows) {
    const int d = bp.dim;
    const int groups = 256 / LPR;
    if (!long_rows) {
        int64_t blocks = (g.n_occ + groups - 1) / groups;
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(k_update<LPR>, dim3((unsigned)blocks), dim3(256), 0, st, ws.counters, ws.uniq_keys, ws.seg_start,
                           sorted_vals, ws.grad, tb, d, bp.lr, bp.eps);
        return hipGetLastError();
    }
    int64_t max_units = g.n_occ / kUnit + g.n_occ / (kLongLen + 1) + 1;
    int64_t ublocks = max_units < 2048 ? max_units : 2048;
    hipLaunchKernelGGL(k_long_partial<LPR>, dim3((unsigned)ublocks), dim3(256), sizeof(double) * 4 * 256, st, ws.counters,
                       ws.long_list, ws.unit_start, ws.seg_start, sorted_vals, ws.grad, d, ws.long_partial);
    int64_t fblocks = (g.n_occ / (kLongLen + 1) + groups) / groups;
    if (fblocks > 1024) fblocks = 1024;
    hipLaunchKernelGGL(k_long_final<LPR>, dim3((unsigned)fblocks), dim3(256), 0, st, ws.counters, ws.long_list,
                       ws.unit_start, ws.uniq_keys, ws.long_partial, tb, d, bp.lr, bp.eps);
    return hipGetLastError();
}

int64_t update_long_rows_capacity(int64_t n_occ) { return n_occ / (kLongLen + 1) + 2; }
int64_t update_long_units_capacity(int64_t n_occ) { return n_occ / kUnit + n_occ / (kLongLen + 1) + 2; }

// Index side: which table rows of the batch take the two-level path, and their units.
hipError_t launch_long_plan(hipStream_t st, int64_t n_occ, const Workspace& ws) {
    if (n_occ <= kSmallSortMax) return hipSuccess;      // the single-workgroup sort kernel has done it
    int64_t blocks = (n_occ + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_long_list, dim3((unsigned)blocks), dim3(256), 0, st, ws.counters, ws.seg_start, ws.long_list);
    hipLaunchKernelGGL(k_long_plan, dim3(1), dim3(256), 0, st, ws.counters, ws.long_list, ws.seg_start, ws.unit_start);
    return hipGetLastError();
}

// long_rows = false: the table rows with few gradient rows; true: the others (two-level sums).
// The two touch disjoint table rows and may run at the same time on different streams.
hipError_t launch_update(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws,
                         const uint32_t* sorted_vals, bool long_rows) {
    if (g.n_occ <= 0) return hipSuccess;
    UpdateTables tb;
    tb.E[0] = bp.E_src; tb.S[0] = bp.S_src;
    tb.E[1] = bp.E_dst; tb.S[1] = bp.S_dst;
    tb.E[2] = bp.E_rel; tb.S[2] = bp.S_rel;
    tb.key_base[0] = 0; tb.key_base[1] = bp.key_base_dst; tb.key_base[2] = bp.key_base_rel;
    const int d = bp.dim;
    if (d <= 32) return launch_update_lpr<8>(st, g, bp, ws, sorted_vals, tb, long_rows);
    if (d <= 64) return launch_update_lpr<16>(st, g, bp, ws, sorted_vals, tb, long_rows);
    if (d <= 128) return launch_update_lpr<32>(st, g, bp, ws, sorted_vals, tb, long_rows);
    return launch_update_lpr<64>(st, g, bp, ws, sorted_vals, tb, long_rows);
}

template <int LPR>
static hipError_t launch_update_small_lpr(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws,
                                          const uint32_t* sorted_vals, const UpdateTables& tb, int64_t loss_n) {
    const int groups = 256 / LPR;
    const int row_blocks = (int)((g.n_occ + groups - 1) / groups);
    const int long_blocks = (int)update_long_rows_capacity(g.n_occ);
    hipLaunchKernelGGL(k_update_small<LPR>, dim3((unsigned)(row_blocks + long_blocks + 1)), dim3(256), 0, st, ws.counters,
                       ws.uniq_keys, ws.seg_start, sorted_vals, ws.long_list, ws.grad, tb, bp.dim, bp.lr, bp.eps, row_blocks,
                       ws.loss_partial, loss_n, ws.loss_sum);
    return hipGetLastError();
}

bool update_is_small(const BatchGeom& g) { return g.n_occ > 0 && g.n_occ <= kSmallSortMax; }

// Whole deterministic update of a small batch (update_is_small) and the sum of its loss terms, one launch.
hipError_t launch_update_small(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws,
                               const uint32_t* sorted_vals, int64_t loss_n) {
    UpdateTables tb;
    tb.E[0] = bp.E_src; tb.S[0] = bp.S_src;
    tb.E[1] = bp.E_dst; tb.S[1] = bp.S_dst;
    tb.E[2] = bp.E_rel; tb.S[2] = bp.S_rel;
    tb.key_base[0] = 0; tb.key_base[1] = bp.key_base_dst; tb.key_base[2] = bp.key_base_rel;
    const int d = bp.dim;
    if (d <= 32) return launch_update_small_lpr<8>(st, g, bp, ws, sorted_vals, tb, loss_n);
    if (d <= 64) return launch_update_small_lpr<16>(st, g, bp, ws, sorted_vals, tb, loss_n);
    if (d <= 128) return launch_update_small_lpr<32>(st, g, bp, ws, sorted_vals, tb, loss_n);
    return launch_update_small_lpr<64>(st, g, bp, ws, sorted_vals, tb, loss_n);
}

// Atomic mode: the batch gradient of every table row already sits in a dense fp32 accumulator
// (summed by hardware float atomics in arrival order); one group per unique row applies
// Adagrad and clears the accumulator row for the next batch.
template <int LPR>
__global__ void __launch_bounds__(256)
k_update_atomic(const uint32_t* __restrict__ counters, const uint32_t* __restrict__ uniq_keys, UpdateTables tb,
                float* G0, float* G1, float* G2, int d, float lr, float eps) {
    const int groups_per_block = 256 / LPR;
    const int gl = threadIdx.x / LPR;
    const int col4 = threadIdx.x % LPR;
    const int c0 = col4 * 4;
    const bool vec4 = (d & 3) == 0;
    const uint32_t n_unique = counters[0];
    for (uint32_t u = blockIdx.x * groups_per_block + gl; u < n_unique; u += gridDim.x * groups_per_block) {
        const uint32_t key = uniq_keys[u];
        const int t = table_of_key(tb, key);
        const int64_t row = (int64_t)(key - tb.key_base[t]);
        for (int cc = c0; cc < d; cc += 4 * LPR) {
            float* gp = (t == 0 ? G0 : t == 1 ? G1 : G2) + row * d + cc;
            double acc[4] = {0.0, 0.0, 0.0, 0.0};
            if (vec4) {
                const float4 v = *reinterpret_cast<const float4*>(gp);
                acc[0] = v.x; acc[1] = v.y; acc[2] = v.z; acc[3] = v.w;
                *reinterpret_cast<float4*>(gp) = make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                for (int j = 0; j < 4 && cc + j < d; ++j) { acc[j] = gp[j]; gp[j] = 0.f; }
            }
            apply_row(tb, key, acc, d, cc, vec4, lr, eps);
        }
    }
}

hipError_t launch_update_atomic(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    if (g.n_occ <= 0) return hipSuccess;
    UpdateTables tb;
    tb.E[0] = bp.E_src; tb.S[0] = bp.S_src;
    tb.E[1] = bp.E_dst; tb.S[1] = bp.S_dst;
    tb.E[2] = bp.E_rel; tb.S[2] = bp.S_rel;
    tb.key_base[0] = 0; tb.key_base[1] = bp.key_base_dst; tb.key_base[2] = bp.key_base_rel;
    const int d = bp.dim;
    const int lpr = d <= 32 ? 8 : d <= 64 ? 16 : d <= 128 ? 32 : 64;
    const int groups = 256 / lpr;
    int64_t blocks = (g.n_occ + groups - 1) / groups;
    if (blocks > 8192) blocks = 8192;
    dim3 grid((unsigned)blocks), block(256);
    switch (lpr) {
        case 8:  hipLaunchKernelGGL(k_update_atomic<8>, grid, block, 0, st, ws.counters, ws.uniq_keys, tb, bp.G_src, bp.G_dst, bp.G_rel, d, bp.lr, bp.eps); break;
        case 16: hipLaunchKernelGGL(k_update_atomic<16>, grid, block, 0, st, ws.counters, ws.uniq_keys, tb, bp.G_src, bp.G_dst, bp.G_rel, d, bp.lr, bp.eps); break;
        case 32: hipLaunchKernelGGL(k_update_atomic<32>, grid, block, 0, st, ws.counters, ws.uniq_keys, tb, bp.G_src, bp.G_dst, bp.G_rel, d, bp.lr, bp.eps); break;
        default: hipLaunchKernelGGL(k_update_atomic<64>, grid, block, 0, st, ws.counters, ws.uniq_keys, tb, bp.G_src, bp.G_dst, bp.G_rel, d, bp.lr, bp.eps); break;
    }
    return hipGetLastError();
}

// ---- f(theta_s, theta_r, theta_d) for global ids: one wavefront per triple ------------------
__global__ void __launch_bounds__(256)
k_score(const int64_t* __restrict__ src, const int32_t* __restrict__ rel, const int64_t* __restrict__ dst,
        int64_t m, float* const* __restrict__ part_emb, int32_t rows_pp, int32_t nparts, int64_t num_nodes,
        const float* __restrict__ E_rel, int32_t num_rel, int32_t d, int32_t score, float* __restrict__ out,
        uint32_t* __restrict__ err_flag) {
    const int lane = lane_id();
    int64_t e = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (e >= m) return;
    int64_t s = src[e], t = dst[e];
    int32_t r = rel ? rel[e] : 0;
    bool bad = s < 0 || s >= num_nodes || t < 0 || t >= num_nodes;
    if (score != LEGEND_SCORE_DOT) bad |= r < 0 || r >= num_rel;
    const float* sp = nullptr;
    const float* tp = nullptr;
    if (!bad) {
        sp = part_emb[s / rows_pp];
        tp = part_emb[t / rows_pp];
    }
    if (bad) { if (lane == 0) { atomicOr(err_flag, 1u); out[e] = 0.f; } return; }
    if (!sp || !tp) { if (lane == 0) { atomicOr(err_flag, 2u); out[e] = 0.f; } return; }
    sp += (s % rows_pp) * d;
    tp += (t % rows_pp) * d;
    const float* rp = E_rel + (int64_t)r * d;
    float acc = 0.f;
    if (score == LEGEND_SCORE_COMPLEX) {
        const int h = d >> 1;
        for (int k = lane; k < h; k += kWave) {
            float qr = sp[k] * rp[k] - sp[k + h] * rp[k + h];
            float qi = sp[k] * rp[k + h] + sp[k + h] * rp[k];
            acc += qr * tp[k] + qi * tp[k + h];
        }
    } else if (score == LEGEND_SCORE_TRANSE_L1) {
        for (int k = lane; k < d; k += kWave) acc -= fabsf((sp[k] + rp[k]) - tp[k]);
    } else if (score == LEGEND_SCORE_DISTMULT) {
        for (int k = lane; k < d; k += kWave) acc += sp[k] * rp[k] * tp[k];
    } else {
        for (int k = lane; k < d; k += kWave) acc += sp[k] * tp[k];
    }
    for (int off = kWave / 2; off > 0; off >>= 1) acc += __shfl_down(acc, off, kWave);
    if (lane == 0) out[e] = acc;
}

hipError_t launch_score(hipStream_t st, const int64_t* src, const int32_t* rel, const int64_t* dst, int64_t m,
                        float* const* part_emb, int32_t rows_per_partition, int32_t num_partitions,
                        int64_t num_nodes, const float* E_rel, int32_t num_relations, int32_t dim,
                        int32_t score, float* out, uint32_t* err_flag) {
    if (m <= 0) return hipSuccess;
    int64_t blocks = (m + 3) / 4;
    hipLaunchKernelGGL(k_score, dim3((unsigned)blocks), dim3(256), 0, st, src, rel, dst, m, part_emb,
                       rows_per_partition, num_partitions, num_nodes, E_rel, num_relations, dim, score, out, err_flag);
    return hipGetLastError();
}

// ---- row gather for reads: rows of non-resident partitions are left untouched ---------------
__global__ void __launch_bounds__(256)
k_gather_rows(const int64_t* __restrict__ ids, int64_t m, float* const* __restrict__ part_base, int32_t rows_pp,
              int64_t num_rows, int32_t d, float* __restrict__ out, uint32_t* __restrict__ err_flag) {
    const int lane = lane_id();
    int64_t e = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (e >= m) return;
    int64_t id = ids[e];
    if (id < 0 || id >= num_rows) { if (lane == 0) atomicOr(err_flag, 1u); return; }
    const float* base = part_base[id / rows_pp];
    if (!base) return;
    const float* p = base + (id % rows_pp) * d;
    for (int k = lane; k < d; k += kWave) out[e * d + k] = p[k];
}

hipError_t launch_gather_rows(hipStream_t st, const int64_t* ids, int64_t m, float* const* part_base,
                              int32_t rows_per_partition, int64_t num_rows, int32_t dim, float* out,
                              uint32_t* err_flag) {
    if (m <= 0) return hipSuccess;
    int64_t blocks = (m + 3) / 4;
    hipLaunchKernelGGL(k_gather_rows, dim3((unsigned)blocks), dim3(256), 0, st, ids, m, part_base,
                       rows_per_partition, num_rows, dim, out, err_flag);
    return hipGetLastError();
}

}  // namespace legend
