// Link-prediction ranks (Sec. 7 "Metrics": MRR and Hits@k are functions of these ranks).
//
// A test triple's corrupted endpoint is replaced by every candidate node; with the score in the
// form (theta_s (x) theta_r) (+) theta_d of Sec. 6 the scores of all replacements are one real
// matrix product: rows q_e = theta_s (x) theta_r (destination side) or conj(theta_r) (x) theta_d
// (source side) against the candidates' embedding rows.  The product runs on 16x16x4 fp32 MFMA
// blocks and is never stored: each block of scores is compared with the triples' own scores and
// only the counts (strictly greater / equal) leave the kernel.
#include <hip/hip_runtime.h>

#include "legend_internal.h"
#include "device_utils.h"

namespace legend {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x4 mfma16(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

constexpr int kRankRows = 64;       // triples per workgroup
constexpr int kRankWaves = 8;
constexpr int kRankSlice = 8;       // k-groups of 16 per register slice of a candidate row

__host__ __device__ inline int rank_dpad(int d) { return (d + 15) & ~15; }
__host__ __device__ inline int rank_stride(int d) { return rank_dpad(d) + 4; }

// ---- q_e, f_e and the true endpoint of every triple: one wavefront per triple ----------------
__global__ void __launch_bounds__(256)
k_rank_compose(const int64_t* __restrict__ src, const int32_t* __restrict__ rel, const int64_t* __restrict__ dst,
               int64_t m, int64_t m_pad, int32_t side, float* const* __restrict__ part_emb, int32_t rows_pp,
               int64_t num_nodes, const float* __restrict__ E_rel, int32_t num_rel, int32_t d, int32_t score,
               float* __restrict__ Q, float* __restrict__ f, int32_t* __restrict__ true_id,
               uint32_t* __restrict__ err_flag) {
    const int lane = lane_id();
    const int64_t e = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (e >= m_pad) return;
    const int dp = rank_dpad(d);
    float* q = Q + e * dp;
    const float* sp = nullptr;
    const float* tp = nullptr;
    int32_t r = 0;
    int64_t s = 0, t = 0;
    bool ok = e < m;
    if (ok) {
        s = src[e]; t = dst[e];
        r = rel ? rel[e] : 0;
        bool bad = s < 0 || s >= num_nodes || t < 0 || t >= num_nodes;
        if (score != LEGEND_SCORE_DOT) bad |= r < 0 || r >= num_rel;
        if (bad) { if (lane == 0) atomicOr(err_flag, 1u); ok = false; }
    }
    if (ok) {
        sp = part_emb[s / rows_pp];
        tp = part_emb[t / rows_pp];
        if (!sp || !tp) { if (lane == 0) atomicOr(err_flag, 2u); ok = false; }
    }
    if (!ok) {
        for (int k = lane; k < dp; k += kWave) q[k] = 0.f;
        if (lane == 0) { f[e] = 0.f; true_id[e] = -1; }
        return;
    }
    sp += (s % rows_pp) * d;
    tp += (t % rows_pp) * d;
    const float* rp = E_rel + (int64_t)r * d;
    // a = the endpoint that stays, b = the endpoint that is replaced
    const float* a = side == LEGEND_CORRUPT_SRC ? tp : sp;
    const float* b = side == LEGEND_CORRUPT_SRC ? sp : tp;
    float acc = 0.f;
    if (score == LEGEND_SCORE_COMPLEX) {
        const int h = d >> 1;
        for (int k = lane; k < h; k += kWave) {
            float qr, qi;
            if (side == LEGEND_CORRUPT_SRC) {   // conj(r) * d
                qr = rp[k] * a[k] + rp[k + h] * a[k + h];
                qi = rp[k] * a[k + h] - rp[k + h] * a[k];
            } else {                            // s * r
                qr = a[k] * rp[k] - a[k + h] * rp[k + h];
                qi = a[k] * rp[k + h] + a[k + h] * rp[k];
            }
            q[k] = qr; q[k + h] = qi;
            acc += qr * b[k] + qi * b[k + h];
        }
    } else if (score == LEGEND_SCORE_TRANSE_L1) {
        for (int k = lane; k < d; k += kWave) {       // s + r meets d; d - r meets s
            const float v = side == LEGEND_CORRUPT_SRC ? a[k] - rp[k] : a[k] + rp[k];
            q[k] = v;
            acc -= fabsf(v - b[k]);
        }
    } else {
        for (int k = lane; k < d; k += kWave) {
            const float v = score == LEGEND_SCORE_DISTMULT ? a[k] * rp[k] : a[k];
            q[k] = v;
            acc += v * b[k];
        }
    }
    for (int k = d + lane; k < dp; k += kWave) q[k] = 0.f;
    for (int off = kWave / 2; off > 0; off >>= 1) acc += __shfl_down(acc, off, kWave);
    if (lane == 0) { f[e] = acc; true_id[e] = (int32_t)(side == LEGEND_CORRUPT_SRC ? s : t); }
}

// Four consecutive components k..k+3 of a candidate row (zeros past the row's end).
template <bool ALIGNED>
__device__ inline float4 cand_load4(const float* __restrict__ row, int k, int d) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (!row) return v;
    if (ALIGNED) {
        if (k < d) v = *reinterpret_cast<const float4*>(row + k);
    } else {
        if (k < d) v.x = row[k];
        if (k + 1 < d) v.y = row[k + 1];
        if (k + 2 < d) v.z = row[k + 2];
        if (k + 3 < d) v.w = row[k + 3];
    }
    return v;
}

// Workgroup (x, y): 64 triples (tile x) against the y-th share of the candidates.  The q rows of
// the tile stay in LDS; wave w takes the blocks of 16 candidates w, w + 8, ... of the share and
// reads their rows straight from the embedding tables into MFMA operands (each row is used by
// exactly one wave of the workgroup, so staging it in LDS would buy nothing).  Operand mapping:
// the contraction index runs in groups of 16; lanes 16g..16g+15 hold components 16G+4g..+3 of
// their row (one 128-bit read) and the s-th of four MFMAs consumes component s of both operands.
template <bool ALIGNED>
__global__ void __launch_bounds__(kRankWaves* kWave, 4)
k_rank(const float* __restrict__ Q, const float* __restrict__ f, const int32_t* __restrict__ true_id, int64_t m,
       const int64_t* __restrict__ cand, int64_t n_cand, int64_t cand_per_wg, float* const* __restrict__ part_emb,
       int32_t rows_pp, int64_t num_nodes, int32_t d, int32_t* __restrict__ greater, int32_t* __restrict__ equal,
       uint32_t* __restrict__ err_flag) {
    extern __shared__ __align__(16) float lds[];
    const int dp = rank_dpad(d);
    const int stride = rank_stride(d);
    float* q_s = lds;                                            // [64][stride]
    float* f_s = q_s + kRankRows * stride;                       // [64]
    int32_t* t_s = reinterpret_cast<int32_t*>(f_s + kRankRows);  // [64]
    int32_t* cnt_s = t_s + kRankRows;                            // [64][2]

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int li = lane & 15, g = lane >> 4;
    const int64_t row0 = (int64_t)blockIdx.x * kRankRows;
    for (int idx = tid; idx < kRankRows * (dp / 4); idx += kRankWaves * kWave) {
        const int r = idx / (dp / 4), k4 = idx % (dp / 4);
        *reinterpret_cast<float4*>(q_s + r * stride + 4 * k4) =
            *reinterpret_cast<const float4*>(Q + (row0 + r) * dp + 4 * k4);
    }
    if (tid < kRankRows) {
        f_s[tid] = f[row0 + tid];
        t_s[tid] = true_id[row0 + tid];
        cnt_s[2 * tid] = 0;
        cnt_s[2 * tid + 1] = 0;
    }
    __syncthreads();

    const int64_t c_lo = (int64_t)blockIdx.y * cand_per_wg;
    const int64_t c_hi = c_lo + cand_per_wg < n_cand ? c_lo + cand_per_wg : n_cand;
    const int nG = dp / 16;
    int gt[4][4], eq[4][4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v) { gt[b][v] = 0; eq[b][v] = 0; }

    for (int64_t cb = c_lo + 16 * w; cb < c_hi; cb += 16 * kRankWaves) {
        // this lane's candidate: the row it supplies as B operand is also the column it holds of C
        const int64_t j = cb + li;
        int64_t cid = -1;
        const float* row = nullptr;
        if (j < c_hi) {
            cid = cand ? cand[j] : j;
            if (cid < 0 || cid >= num_nodes) {
                if (g == 0) atomicOr(err_flag, 1u);
                cid = -1;
            } else {
                const float* base = part_emb[cid / rows_pp];
                if (!base) { if (g == 0) atomicOr(err_flag, 2u); cid = -1; }
                else row = base + (cid % rows_pp) * d;
            }
        }
        f32x4 acc[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int G0 = 0; G0 < nG; G0 += kRankSlice) {
            float4 bv[kRankSlice];
#pragma unroll
            for (int u = 0; u < kRankSlice; ++u)
                bv[u] = (G0 + u < nG) ? cand_load4<ALIGNED>(row, 16 * (G0 + u) + 4 * g, d) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < kRankSlice; ++u) {
                if (G0 + u < nG) {
                    const float* qa = q_s + li * stride + 16 * (G0 + u) + 4 * g;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const float4 av = *reinterpret_cast<const float4*>(qa + 16 * b * stride);
                        acc[b] = mfma16(av.x, bv[u].x, acc[b]);
                        acc[b] = mfma16(av.y, bv[u].y, acc[b]);
                        acc[b] = mfma16(av.z, bv[u].z, acc[b]);
                        acc[b] = mfma16(av.w, bv[u].w, acc[b]);
                    }
                }
            }
        }
        // C layout: acc[b][v] = score of triple 16b + 4g + v against this lane's candidate
        const int32_t cid32 = (int32_t)cid;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const float4 fr = *reinterpret_cast<const float4*>(f_s + 16 * b + 4 * g);
            const int4 tr = *reinterpret_cast<const int4*>(t_s + 16 * b + 4 * g);
            const float fv[4] = {fr.x, fr.y, fr.z, fr.w};
            const int tv[4] = {tr.x, tr.y, tr.z, tr.w};
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool counted = cid >= 0 && cid32 != tv[v];
                gt[b][v] += (counted && acc[b][v] > fv[v]) ? 1 : 0;
                eq[b][v] += (counted && acc[b][v] == fv[v]) ? 1 : 0;
            }
        }
    }
    // the 16 lanes of a lane group hold different candidates of the same 16 triples
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            int a = gt[b][v], e = eq[b][v];
#pragma unroll
            for (int mask = 1; mask < 16; mask <<= 1) {
                a += __shfl_xor(a, mask, kWave);
                e += __shfl_xor(e, mask, kWave);
            }
            if (li == 0) {
                if (a) atomicAdd(&cnt_s[2 * (16 * b + 4 * g + v)], a);
                if (e) atomicAdd(&cnt_s[2 * (16 * b + 4 * g + v) + 1], e);
            }
        }
    __syncthreads();
    if (tid < kRankRows && row0 + tid < m) {
        if (cnt_s[2 * tid]) atomicAdd(&greater[row0 + tid], cnt_s[2 * tid]);
        if (cnt_s[2 * tid + 1]) atomicAdd(&equal[row0 + tid], cnt_s[2 * tid + 1]);
    }
}

// The same counts for the translational score -|q - c|_1: no matrix product.  A lane keeps one
// candidate row in registers (dim <= 128) and meets the 64 q rows of the tile one after the other
// (LDS broadcast reads); the comparisons of a row against 64 candidates are counted by ballot.
constexpr int kRankTransWaves = 4;
constexpr int kRankTransMaxD4 = 32;

template <bool ALIGNED>
__global__ void __launch_bounds__(kRankTransWaves* kWave)
k_rank_trans(const float* __restrict__ Q, const float* __restrict__ f, const int32_t* __restrict__ true_id, int64_t m,
             const int64_t* __restrict__ cand, int64_t n_cand, int64_t cand_per_wg, float* const* __restrict__ part_emb,
             int32_t rows_pp, int64_t num_nodes, int32_t d, int32_t* __restrict__ greater, int32_t* __restrict__ equal,
             uint32_t* __restrict__ err_flag) {
    extern __shared__ __align__(16) float lds[];
    const int dp = rank_dpad(d);
    const int stride = rank_stride(d);
    float* q_s = lds;
    float* f_s = q_s + kRankRows * stride;
    int32_t* t_s = reinterpret_cast<int32_t*>(f_s + kRankRows);
    int32_t* cnt_s = t_s + kRankRows;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * kRankRows;
    for (int idx = tid; idx < kRankRows * (dp / 4); idx += kRankTransWaves * kWave) {
        const int r = idx / (dp / 4), k4 = idx % (dp / 4);
        *reinterpret_cast<float4*>(q_s + r * stride + 4 * k4) =
            *reinterpret_cast<const float4*>(Q + (row0 + r) * dp + 4 * k4);
    }
    if (tid < kRankRows) {
        f_s[tid] = f[row0 + tid];
        t_s[tid] = true_id[row0 + tid];
        cnt_s[2 * tid] = 0;
        cnt_s[2 * tid + 1] = 0;
    }
    __syncthreads();
    const int64_t c_lo = (int64_t)blockIdx.y * cand_per_wg;
    const int64_t c_hi = c_lo + cand_per_wg < n_cand ? c_lo + cand_per_wg : n_cand;
    const int d4 = (d + 3) >> 2;
    const int nrows = (int)(m - row0 < kRankRows ? m - row0 : kRankRows);
    for (int64_t cb = c_lo + kWave * w; cb < c_hi; cb += kWave * kRankTransWaves) {
        const int64_t j = cb + lane;
        int64_t cid = -1;
        const float* row = nullptr;
        if (j < c_hi) {
            cid = cand ? cand[j] : j;
            if (cid < 0 || cid >= num_nodes) {
                atomicOr(err_flag, 1u);
                cid = -1;
            } else {
                const float* base = part_emb[cid / rows_pp];
                if (!base) { atomicOr(err_flag, 2u); cid = -1; }
                else row = base + (cid % rows_pp) * d;
            }
        }
        float4 cr[kRankTransMaxD4];
#pragma unroll
        for (int j4 = 0; j4 < kRankTransMaxD4; ++j4)
            cr[j4] = j4 < d4 ? cand_load4<ALIGNED>(row, 4 * j4, d) : make_float4(0.f, 0.f, 0.f, 0.f);
        const int32_t cid32 = (int32_t)cid;
        for (int r = 0; r < nrows; ++r) {
            const float* qr = q_s + r * stride;
            float s = 0.f;
#pragma unroll
            for (int j4 = 0; j4 < kRankTransMaxD4; ++j4) {
                if (j4 < d4) {
                    const float4 q4 = *reinterpret_cast<const float4*>(qr + 4 * j4);
                    s += (fabsf(q4.x - cr[j4].x) + fabsf(q4.y - cr[j4].y)) + (fabsf(q4.z - cr[j4].z) + fabsf(q4.w - cr[j4].w));
                }
            }
            const float S = -s, fv = f_s[r];
            const bool counted = cid >= 0 && cid32 != t_s[r];
            const unsigned long long gtm = __ballot(counted && S > fv), eqm = __ballot(counted && S == fv);
            if (lane == 0) {
                if (gtm) atomicAdd(&cnt_s[2 * r], __popcll(gtm));
                if (eqm) atomicAdd(&cnt_s[2 * r + 1], __popcll(eqm));
            }
        }
    }
    __syncthreads();
    if (tid < kRankRows && row0 + tid < m) {
        if (cnt_s[2 * tid]) atomicAdd(&greater[row0 + tid], cnt_s[2 * tid]);
        if (cnt_s[2 * tid + 1]) atomicAdd(&equal[row0 + tid], cnt_s[2 * tid + 1]);
    }
}

// rank = 1 + greater + equal / 2;  sums of 1/rank and of the hit indicators in a fixed order
__global__ void __launch_bounds__(256)
k_rank_metrics(const int32_t* __restrict__ greater, const int32_t* __restrict__ equal, int64_t m,
               double* __restrict__ out /* [4]: mrr, hits@1, hits@3, hits@10 */) {
    __shared__ double part[4][256];
    double s[4] = {0.0, 0.0, 0.0, 0.0};
    for (int64_t e = threadIdx.x; e < m; e += 256) {
        const double rank = 1.0 + (double)greater[e] + 0.5 * (double)equal[e];
        s[0] += 1.0 / rank;
        s[1] += rank <= 1.0 ? 1.0 : 0.0;
        s[2] += rank <= 3.0 ? 1.0 : 0.0;
        s[3] += rank <= 10.0 ? 1.0 : 0.0;
    }
    for (int k = 0; k < 4; ++k) part[k][threadIdx.x] = s[k];
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off)
            for (int k = 0; k < 4; ++k) part[k][threadIdx.x] += part[k][threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x < 4) out[threadIdx.x] = m > 0 ? part[threadIdx.x][0] / (double)m : 0.0;
}

}  // namespace

int64_t rank_rows_padded(int64_t m) { return (m + kRankRows - 1) / kRankRows * kRankRows; }
int rank_dim_padded(int d) { return rank_dpad(d); }

hipError_t launch_rank(hipStream_t st, const int64_t* src, const int32_t* rel, const int64_t* dst, int64_t m,
                       int32_t side, const int64_t* cand, int64_t n_cand, float* const* part_emb,
                       int32_t rows_per_partition, int64_t num_nodes, const float* E_rel, int32_t num_relations,
                       int32_t dim, int32_t score, float* Q, float* f, int32_t* true_id, int32_t* greater,
                       int32_t* equal, double* metrics, uint32_t* err_flag) {
    if (m <= 0) return hipSuccess;
    const int64_t m_pad = rank_rows_padded(m);
    hipLaunchKernelGGL(k_rank_compose, dim3((unsigned)((m_pad + 3) / 4)), dim3(256), 0, st, src, rel, dst, m, m_pad, side,
                       part_emb, rows_per_partition, num_nodes, E_rel, num_relations, dim, score, Q, f, true_id, err_flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (n_cand > 0) {
        const int64_t tiles = m_pad / kRankRows;
        const bool aligned = dim % 4 == 0;
        const size_t lds = sizeof(float) * ((size_t)kRankRows * rank_stride(dim) + kRankRows) + sizeof(int32_t) * 3 * kRankRows;
        if (score == LEGEND_SCORE_TRANSE_L1) {
            if (dim > 4 * kRankTransMaxD4) return hipErrorInvalidValue;
            const int64_t step = kWave * kRankTransWaves;
            int64_t shares = (4096 + tiles - 1) / tiles;
            const int64_t max_shares = (n_cand + step - 1) / step;
            if (shares > max_shares) shares = max_shares;
            if (shares < 1) shares = 1;
            if (shares > 65535) shares = 65535;
            int64_t per = (n_cand + shares - 1) / shares;
            per = (per + step - 1) / step * step;
            shares = (n_cand + per - 1) / per;
            const void* fn = aligned ? reinterpret_cast<const void*>(&k_rank_trans<true>) : reinterpret_cast<const void*>(&k_rank_trans<false>);
            e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            dim3 grid((unsigned)tiles, (unsigned)shares), block(kRankTransWaves * kWave);
            if (aligned)
                hipLaunchKernelGGL(k_rank_trans<true>, grid, block, lds, st, Q, f, true_id, m, cand, n_cand, per, part_emb,
                                   rows_per_partition, num_nodes, dim, greater, equal, err_flag);
            else
                hipLaunchKernelGGL(k_rank_trans<false>, grid, block, lds, st, Q, f, true_id, m, cand, n_cand, per, part_emb,
                                   rows_per_partition, num_nodes, dim, greater, equal, err_flag);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(k_rank_metrics, dim3(1), dim3(256), 0, st, greater, equal, m, metrics);
            return hipGetLastError();
        }
        // enough workgroups to fill the chip a few times over, each with at least four blocks per wave
        const int64_t min_share = 16 * kRankWaves * 4;
        int64_t shares = (4096 + tiles - 1) / tiles;
        const int64_t max_shares = (n_cand + min_share - 1) / min_share;
        if (shares > max_shares) shares = max_shares;
        if (shares < 1) shares = 1;
        if (shares > 65535) shares = 65535;
        int64_t per = (n_cand + shares - 1) / shares;
        per = (per + 16 * kRankWaves - 1) / (16 * kRankWaves) * (16 * kRankWaves);
        shares = (n_cand + per - 1) / per;
        const void* fn = aligned ? reinterpret_cast<const void*>(&k_rank<true>) : reinterpret_cast<const void*>(&k_rank<false>);
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        dim3 grid((unsigned)tiles, (unsigned)shares), block(kRankWaves * kWave);
        if (aligned)
            hipLaunchKernelGGL(k_rank<true>, grid, block, lds, st, Q, f, true_id, m, cand, n_cand, per, part_emb,
                               rows_per_partition, num_nodes, dim, greater, equal, err_flag);
        else
            hipLaunchKernelGGL(k_rank<false>, grid, block, lds, st, Q, f, true_id, m, cand, n_cand, per, part_emb,
                               rows_per_partition, num_nodes, dim, greater, equal, err_flag);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_rank_metrics, dim3(1), dim3(256), 0, st, greater, equal, m, metrics);
    return hipGetLastError();
}

}  // namespace legend
