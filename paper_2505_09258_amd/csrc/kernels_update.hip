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

// LPR lanes (a float4 each) own one table row.
template <int LPR>
__global__ void __launch_bounds__(256)
k_update(const uint32_t* __restrict__ counters, const uint32_t* __restrict__ uniq_keys,
         const uint32_t* __restrict__ seg_start, const uint32_t* __restrict__ sorted_vals,
         const float* __restrict__ grad, UpdateTables tb, int d, float lr, float eps) {
    const int groups_per_block = 256 / LPR;
    const int gl = threadIdx.x / LPR;
    const int col4 = threadIdx.x % LPR;
    const int c0 = col4 * 4;
    const bool vec4 = (d & 3) == 0;
    const uint32_t n_unique = counters[0];
    for (uint32_t u = blockIdx.x * groups_per_block + gl; u < n_unique; u += gridDim.x * groups_per_block) {
        if (c0 >= d) continue;
        const uint32_t key = uniq_keys[u];
        const int t = key >= tb.key_base[2] ? 2 : (key >= tb.key_base[1] && tb.key_base[1] > 0 ? 1 : 0);
        const int64_t row = (int64_t)(key - tb.key_base[t]);
        const uint32_t lo = seg_start[u], hi = seg_start[u + 1];
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
        for (uint32_t p = lo; p < hi; ++p) {
            const float* gp = grad + (int64_t)sorted_vals[p] * d + c0;
            if (vec4) {
                float4 v = *reinterpret_cast<const float4*>(gp);
                a0 += (double)v.x; a1 += (double)v.y; a2 += (double)v.z; a3 += (double)v.w;
            } else {
                a0 += (double)gp[0];
                if (c0 + 1 < d) a1 += (double)gp[1];
                if (c0 + 2 < d) a2 += (double)gp[2];
                if (c0 + 3 < d) a3 += (double)gp[3];
            }
        }
        float* ep = tb.E[t] + row * d + c0;
        float* sp = tb.S[t] + row * d + c0;
        if (vec4) {
            float4 th = *reinterpret_cast<float4*>(ep);
            float4 st = *reinterpret_cast<float4*>(sp);
            adagrad_elem((float)a0, th.x, st.x, lr, eps);
            adagrad_elem((float)a1, th.y, st.y, lr, eps);
            adagrad_elem((float)a2, th.z, st.z, lr, eps);
            adagrad_elem((float)a3, th.w, st.w, lr, eps);
            *reinterpret_cast<float4*>(ep) = th;
            *reinterpret_cast<float4*>(sp) = st;
        } else {
            double acc[4] = {a0, a1, a2, a3};
            for (int j = 0; j < 4 && c0 + j < d; ++j) {
                float th = ep[j], st = sp[j];
                adagrad_elem((float)acc[j], th, st, lr, eps);
                ep[j] = th;
                sp[j] = st;
            }
        }
    }
}

hipError_t launch_update(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws,
                         const uint32_t* sorted_vals, int32_t rows_per_partition) {
    (void)rows_per_partition;
    if (g.n_occ <= 0) return hipSuccess;
    UpdateTables tb;
    tb.E[0] = bp.E_src; tb.S[0] = bp.S_src;
    tb.E[1] = bp.E_dst; tb.S[1] = bp.S_dst;
    tb.E[2] = bp.E_rel; tb.S[2] = bp.S_rel;
    tb.key_base[0] = 0; tb.key_base[1] = bp.key_base_dst; tb.key_base[2] = bp.key_base_rel;
    const int d = bp.dim;
    int lpr = d <= 32 ? 8 : d <= 64 ? 16 : d <= 128 ? 32 : 64;
    int groups = 256 / lpr;
    int64_t blocks = (g.n_occ + groups - 1) / groups;
    if (blocks > 8192) blocks = 8192;
    dim3 grid((unsigned)blocks), block(256);
    switch (lpr) {
        case 8:  hipLaunchKernelGGL(k_update<8>, grid, block, 0, st, ws.counters, ws.uniq_keys, ws.seg_start, sorted_vals, ws.grad, tb, d, bp.lr, bp.eps); break;
        case 16: hipLaunchKernelGGL(k_update<16>, grid, block, 0, st, ws.counters, ws.uniq_keys, ws.seg_start, sorted_vals, ws.grad, tb, d, bp.lr, bp.eps); break;
        case 32: hipLaunchKernelGGL(k_update<32>, grid, block, 0, st, ws.counters, ws.uniq_keys, ws.seg_start, sorted_vals, ws.grad, tb, d, bp.lr, bp.eps); break;
        default: hipLaunchKernelGGL(k_update<64>, grid, block, 0, st, ws.counters, ws.uniq_keys, ws.seg_start, sorted_vals, ws.grad, tb, d, bp.lr, bp.eps); break;
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
