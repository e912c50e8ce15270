// Batch computation (paper Sec. 2.1 stage 5, Sec. 6): one workgroup per (chunk row tile,
// corrupted side) gathers the rows of its positives, forms Q = theta_s (x) theta_r (or
// its mirror conj(theta_r) (x) theta_d for source-side corruption; the paper's
// "Intermediate Result 1"), the positive scores, and then sweeps the chunk's shared
// negatives in tiles of 64 rows staged through LDS:
//     S = Q * Neg^T                 negative scores        (fp32 MFMA 32x32x2)
//     W = dl/dS                     softmax / logistic     (VALU, in LDS)
//     G_Q += W * Neg                gradient w.r.t. Q      (fp32 MFMA)
//     G_neg = W^T * Q               gradient of negatives  (fp32 MFMA)
// The paper keeps exp(S) in global memory between the forward and backward kernels
// ("Intermediate Result 3"); a 64 x N score block does not fit the 160 KB LDS of a
// CDNA4 compute unit, so for Eq. 1 the sweep runs twice (log-sum-exp first, then the
// gradients with S recomputed) and nothing but gradient rows is ever written to HBM.
// Wavefronts are 64 wide: a 64x64 score tile is four 32x32 MFMA blocks, one per wave.
#include "legend_internal.h"
#include "device_utils.h"

namespace legend {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kChunkThreads = 256;
constexpr int kRowTile = 64;    // positives per workgroup (padded)
constexpr int kNegTile = 64;    // negatives per LDS tile
constexpr int kWS = kNegTile + 1;

int row_tiles_for(int chunk_size) { return (chunk_size + kRowTile - 1) / kRowTile; }
int rows_per_tile_for(int chunk_size) {
    int t = row_tiles_for(chunk_size);
    return (chunk_size + t - 1) / t;
}
int max_dim_supported() { return 128; }

__device__ inline f32x16 mfma32(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ inline float softplusf(float x) {
    // log(1 + exp(x)) without overflow
    return fmaxf(x, 0.f) + log1pf(expf(-fabsf(x)));
}
__device__ inline float sigmoidf(float x) { return 1.f / (1.f + expf(-x)); }

// NB: number of 32-wide column blocks covering the embedding dimension (dim <= 32 * NB).
template <int NB, int SCORE, int LOSS>
__global__ void __launch_bounds__(kChunkThreads)
k_chunk(BatchGeom g, BucketParams bp, const int32_t* __restrict__ neg_ids, float* __restrict__ grad,
        double* __restrict__ loss_partial) {
    constexpr int LPR = NB * 8;             // lanes that cooperate on one gathered row (float4 each)
    constexpr int RPS = kWave / LPR;        // rows a wave gathers per step
    constexpr int STEPS = 16 / RPS;         // each wave gathers 16 of the 64 tile rows
    constexpr int NBW = (2 * NB + 3) / 4;   // 32x32 output blocks per wave in the gradient products

    extern __shared__ float smem[];
    const int d = bp.dim;
    const int QS = (d + 1) | 1;             // odd LDS row stride >= dim rounded up to even
    const int KD = (d + 1) & ~1;
    const int tile_floats = kRowTile * QS + 32 * NB;
    float* Qs = smem;                       // [64][QS]  Q rows of this workgroup
    float* Ns = Qs + tile_floats;           // [64][QS]  current negative tile (later: G_Q)
    float* Ws = Ns + tile_floats;           // [64][65]  S, then W, of the current tile
    float* pos_s = Ws + kRowTile * kWS;     // [64]
    float* rowloss_s = pos_s + kRowTile;    // [64]

    const int tid = threadIdx.x;
    const int w = tid >> 6;
    const int lane = tid & 63;
    const int i32 = lane & 31;
    const int kk = lane >> 5;

    // which piece of the batch
    int wg = blockIdx.x;
    const int t = wg % g.T;  wg /= g.T;
    const int c = wg % g.nchunks;
    const int si = wg / g.nchunks;
    const int side = g.side_id[si];          // 0: destination corrupted, 1: source corrupted
    const int chunk_rows = min(g.C, g.P - c * g.C);
    const int row0 = t * g.rows_tile;
    const int nrows = max(0, min(g.rows_tile, chunk_rows - row0));
    const int64_t e0 = (int64_t)c * g.C + row0;                  // first positive (batch-local)
    const int32_t* eb = bp.edges + (bp.batch_lo + e0) * 3;
    const float* Ex = side == 0 ? bp.E_src : bp.E_dst;          // rows combined with the relation
    const float* Ey = side == 0 ? bp.E_dst : bp.E_src;          // rows that meet Q
    const float* En = Ey;                                        // negatives replace the y endpoint
    const int xcol = side == 0 ? 0 : 2;
    const int ycol = 2 - xcol;
    const int N = g.N;
    const int32_t* my_negs = neg_ids + ((int64_t)si * g.nchunks + c) * N;
    const int64_t side_base = (int64_t)si * g.per_side;
    const int64_t neg_base = side_base + (int64_t)g.roles * g.P + ((int64_t)c * g.T + t) * N;
    const bool vec4 = (d & 3) == 0;

    // ---- zero the pad columns [d, QS) of both row tiles (never written again) -------------
    for (int idx = tid; idx < kRowTile * (QS - d); idx += kChunkThreads) {
        int r = idx / (QS - d), cc = d + idx % (QS - d);
        Qs[r * QS + cc] = 0.f;
        Ns[r * QS + cc] = 0.f;
    }

    // ---- prologue: Q rows and positive scores; 4 threads per row --------------------------
    const int prow = tid >> 2;
    const int ppart = tid & 3;
    {
        float partial = 0.f;
        if (prow < nrows) {
            const float* x = Ex + (int64_t)eb[prow * 3 + xcol] * d;
            const float* y = Ey + (int64_t)eb[prow * 3 + ycol] * d;
            const float* r = SCORE == LEGEND_SCORE_DOT ? x : bp.E_rel + (int64_t)eb[prow * 3 + 1] * d;
            if (SCORE == LEGEND_SCORE_COMPLEX) {
                const int h = d >> 1;
                for (int k = ppart; k < h; k += 4) {
                    float xr = x[k], xi = x[k + h], rr = r[k], ri = r[k + h];
                    float qr, qi;
                    if (side == 0) { qr = xr * rr - xi * ri; qi = xr * ri + xi * rr; }
                    else           { qr = rr * xr + ri * xi; qi = rr * xi - ri * xr; }
                    Qs[prow * QS + k] = qr;
                    Qs[prow * QS + k + h] = qi;
                    partial += qr * y[k] + qi * y[k + h];
                }
            } else {
                for (int k = ppart; k < d; k += 4) {
                    float q = SCORE == LEGEND_SCORE_DOT ? x[k] : x[k] * r[k];
                    Qs[prow * QS + k] = q;
                    partial += q * y[k];
                }
            }
        } else {
            for (int k = ppart; k < d; k += 4) Qs[prow * QS + k] = 0.f;
        }
        partial += wave_shfl_xor(partial, 1);
        partial += wave_shfl_xor(partial, 2);
        if (ppart == 0) pos_s[prow] = partial;
    }

    // ---- negative tile gather: registers first, LDS after the previous tile is done -------
    float4 pf[STEPS];
    const int grow_lane = lane / LPR;         // row within a step
    const int gcol4 = lane % LPR;             // float4 column
    auto gather_issue = [&](int n0) {
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            int rt = w * 16 + s * RPS + grow_lane;
            int k = n0 + rt;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            int c0 = gcol4 * 4;
            if (k < N && c0 < d) {
                const float* p = En + (int64_t)my_negs[k] * d + c0;
                if (vec4) {
                    v = *reinterpret_cast<const float4*>(p);
                } else {
                    v.x = p[0];
                    if (c0 + 1 < d) v.y = p[1];
                    if (c0 + 2 < d) v.z = p[2];
                    if (c0 + 3 < d) v.w = p[3];
                }
            }
            pf[s] = v;
        }
    };
    auto gather_commit = [&]() {
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            int rt = w * 16 + s * RPS + grow_lane;
            int c0 = gcol4 * 4;
            float* dst = Ns + rt * QS + c0;
            if (c0 < d) dst[0] = pf[s].x;
            if (c0 + 1 < d) dst[1] = pf[s].y;
            if (c0 + 2 < d) dst[2] = pf[s].z;
            if (c0 + 3 < d) dst[3] = pf[s].w;
        }
    };

    const int rbA = w & 1, cbA = w >> 1;      // this wave's 32x32 block of the score tile
    auto scores_to_lds = [&]() {
        f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        const float* qa = Qs + (rbA * 32 + i32) * QS + kk;
        const float* nb = Ns + (cbA * 32 + i32) * QS + kk;
        for (int k0 = 0; k0 < KD; k0 += 2) acc = mfma32(qa[k0], nb[k0], acc);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int row = rbA * 32 + 8 * (v >> 2) + 4 * kk + (v & 3);
            Ws[row * kWS + cbA * 32 + i32] = acc[v];
        }
    };

    const int ntiles = (N + kNegTile - 1) / kNegTile;
    const int srow = tid >> 2;                // softmax bookkeeping: 4 threads per row
    const int sq = tid & 3;
    float lse = 0.f;
    float neg_loss = 0.f;                     // logistic: sum of weighted softplus terms

    gather_issue(0);
    __syncthreads();                          // Qs, pos_s complete

    if (LOSS == LEGEND_LOSS_SOFTMAX) {
        // ---- sweep 1: running max and sum of exp per row ------------------------------------
        float m_run = -INFINITY, l_run = 0.f;
        for (int tile = 0; tile < ntiles; ++tile) {
            const int n0 = tile * kNegTile;
            gather_commit();
            __syncthreads();
            gather_issue(tile + 1 < ntiles ? n0 + kNegTile : 0);   // next tile, or first tile of sweep 2
            scores_to_lds();
            __syncthreads();
            const float* wr = Ws + srow * kWS + sq * 16;
            const int ncol = min(16, N - n0 - sq * 16);            // valid columns of my 16
            float tmax = -INFINITY;
            for (int j = 0; j < ncol; ++j) tmax = fmaxf(tmax, wr[j]);
            tmax = fmaxf(tmax, wave_shfl_xor(tmax, 1));
            tmax = fmaxf(tmax, wave_shfl_xor(tmax, 2));
            float m_new = fmaxf(m_run, tmax);
            float sum = 0.f;
            for (int j = 0; j < ncol; ++j) sum += expf(wr[j] - m_new);
            sum += wave_shfl_xor(sum, 1);
            sum += wave_shfl_xor(sum, 2);
            l_run = l_run * expf(m_run - m_new) + sum;
            m_run = m_new;
        }
        lse = m_run + logf(l_run);
    }

    // ---- sweep 2: gradients ----------------------------------------------------------------
    f32x16 accB[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) accB[j][v] = 0.f;
    const int rbG = w & 1;
    const int rows2 = (nrows + 1) & ~1;
    const float wneg = bp.neg_weight;

    for (int tile = 0; tile < ntiles; ++tile) {
        const int n0 = tile * kNegTile;
        gather_commit();
        __syncthreads();
        if (tile + 1 < ntiles) gather_issue(n0 + kNegTile);
        scores_to_lds();
        __syncthreads();
        {
            float* wr = Ws + srow * kWS + sq * 16;
            const int ncol = srow < nrows ? min(16, N - n0 - sq * 16) : 0;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                float s = wr[j];
                float wv = 0.f;
                if (j < ncol) {
                    if (LOSS == LEGEND_LOSS_SOFTMAX) {
                        wv = expf(s - lse);
                    } else {
                        wv = wneg * sigmoidf(s);
                        neg_loss += wneg * softplusf(s);
                    }
                }
                wr[j] = wv;
            }
        }
        __syncthreads();
        const int kmax = min(kNegTile, (N - n0 + 1) & ~1);
        // G_Q += W * Neg
        {
            const float* wa = Ws + (rbG * 32 + i32) * kWS + kk;
            const float* nb = Ns + kk * QS + i32;
            for (int k0 = 0; k0 < kmax; k0 += 2) {
                float a = wa[k0];
#pragma unroll
                for (int j = 0; j < NBW; ++j) {
                    int cb = (w >> 1) + 2 * j;
                    if (cb < NB) accB[j] = mfma32(a, nb[k0 * QS + cb * 32], accB[j]);
                }
            }
        }
        // G_neg = W^T * Q, written straight to the staged gradient rows
        {
            f32x16 accC[NBW];
#pragma unroll
            for (int j = 0; j < NBW; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) accC[j][v] = 0.f;
            const float* wa = Ws + kk * kWS + rbG * 32 + i32;
            const float* qb = Qs + kk * QS + i32;
            for (int k0 = 0; k0 < rows2; k0 += 2) {
                float a = wa[k0 * kWS];
#pragma unroll
                for (int j = 0; j < NBW; ++j) {
                    int cb = (w >> 1) + 2 * j;
                    if (cb < NB) accC[j] = mfma32(a, qb[k0 * QS + cb * 32], accC[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < NBW; ++j) {
                int cb = (w >> 1) + 2 * j;
                int col = cb * 32 + i32;
                if (cb < NB && col < d) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        int neg = n0 + rbG * 32 + 8 * (v >> 2) + 4 * kk + (v & 3);
                        if (neg < N) grad[(neg_base + neg) * d + col] = accC[j][v];
                    }
                }
            }
        }
        __syncthreads();
    }

    // ---- epilogue: G_Q to LDS, chain rule, gradient rows of the positives -------------------
    float* Gs = Ns;
#pragma unroll
    for (int j = 0; j < NBW; ++j) {
        int cb = (w >> 1) + 2 * j;
        int col = cb * 32 + i32;
        if (cb < NB && col < d) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int row = rbG * 32 + 8 * (v >> 2) + 4 * kk + (v & 3);
                Gs[row * QS + col] = accB[j][v];
            }
        }
    }
    __syncthreads();
    {
        float row_loss = 0.f;
        if (LOSS == LEGEND_LOSS_LOGISTIC) {
            neg_loss += wave_shfl_xor(neg_loss, 1);
            neg_loss += wave_shfl_xor(neg_loss, 2);
        }
        if (prow < nrows) {
            const float f = pos_s[prow];
            float a;
            if (LOSS == LEGEND_LOSS_SOFTMAX) { a = -1.f; row_loss = lse - f; }
            else { a = -sigmoidf(-f); row_loss = softplusf(-f) + neg_loss; }
            const float* x = Ex + (int64_t)eb[prow * 3 + xcol] * d;
            const float* y = Ey + (int64_t)eb[prow * 3 + ycol] * d;
            const float* r = SCORE == LEGEND_SCORE_DOT ? x : bp.E_rel + (int64_t)eb[prow * 3 + 1] * d;
            const int64_t e = e0 + prow;
            float* gx = grad + (side_base + (side == 0 ? 0 : g.P) + e) * d;        // source rows first
            float* gy = grad + (side_base + (side == 0 ? g.P : 0) + e) * d;
            float* gr = grad + (side_base + 2 * (int64_t)g.P + e) * d;
            const float* gq = Gs + prow * QS;
            const float* q = Qs + prow * QS;
            if (SCORE == LEGEND_SCORE_COMPLEX) {
                const int h = d >> 1;
                for (int k = ppart; k < h; k += 4) {
                    float gre = gq[k] + a * y[k], gim = gq[k + h] + a * y[k + h];
                    float xr = x[k], xi = x[k + h], rr = r[k], ri = r[k + h];
                    gy[k] = a * q[k];
                    gy[k + h] = a * q[k + h];
                    if (side == 0) {
                        gx[k] = rr * gre + ri * gim;      gx[k + h] = rr * gim - ri * gre;   // conj(r) g
                        gr[k] = xr * gre + xi * gim;      gr[k + h] = xr * gim - xi * gre;   // conj(x) g
                    } else {
                        gx[k] = rr * gre - ri * gim;      gx[k + h] = rr * gim + ri * gre;   // r g
                        gr[k] = gre * xr + gim * xi;      gr[k + h] = gre * xi - gim * xr;   // conj(g) x
                    }
                }
            } else {
                for (int k = ppart; k < d; k += 4) {
                    float gv = gq[k] + a * y[k];
                    gy[k] = a * q[k];
                    if (SCORE == LEGEND_SCORE_DOT) {
                        gx[k] = gv;
                    } else {
                        gx[k] = r[k] * gv;
                        gr[k] = x[k] * gv;
                    }
                }
            }
        }
        if (ppart == 0) rowloss_s[prow] = row_loss;
    }
    __syncthreads();
    if (tid == 0) {
        double s = 0.0;
        for (int r = 0; r < kRowTile; ++r) s += (double)rowloss_s[r];
        loss_partial[blockIdx.x] = s;
    }
}

static size_t chunk_lds_bytes(int d, int nb) {
    int QS = (d + 1) | 1;
    size_t floats = 2 * ((size_t)kRowTile * QS + 32 * nb) + (size_t)kRowTile * kWS + 2 * kRowTile;
    return floats * sizeof(float);
}

template <int NB>
static hipError_t launch_chunks_nb(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    dim3 grid((unsigned)(g.sides * g.nchunks * g.T)), block(kChunkThreads);
    size_t lds = chunk_lds_bytes(bp.dim, NB);
#define LEGEND_CHUNK_CASE(SC, LO)                                                                              \
    if (bp.score == SC && bp.loss == LO) {                                                                     \
        static size_t lds_allowed = 0; /* dynamic LDS above 64 KB has to be requested per kernel */            \
        if (lds > lds_allowed) {                                                                               \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_chunk<NB, SC, LO>),            \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
            if (e != hipSuccess) return e;                                                                     \
            lds_allowed = lds;                                                                                 \
        }                                                                                                      \
        hipLaunchKernelGGL((k_chunk<NB, SC, LO>), grid, block, lds, st, g, bp, ws.neg_ids, ws.grad,            \
                           ws.loss_partial);                                                                   \
        return hipGetLastError();                                                                              \
    }
    LEGEND_CHUNK_CASE(LEGEND_SCORE_DOT, LEGEND_LOSS_SOFTMAX)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_DOT, LEGEND_LOSS_LOGISTIC)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_DISTMULT, LEGEND_LOSS_SOFTMAX)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_DISTMULT, LEGEND_LOSS_LOGISTIC)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_COMPLEX, LEGEND_LOSS_SOFTMAX)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_COMPLEX, LEGEND_LOSS_LOGISTIC)
#undef LEGEND_CHUNK_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_chunks(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    if (g.P <= 0) return hipSuccess;
    if (bp.dim <= 32) return launch_chunks_nb<1>(st, g, bp, ws);
    if (bp.dim <= 64) return launch_chunks_nb<2>(st, g, bp, ws);
    if (bp.dim <= 128) return launch_chunks_nb<4>(st, g, bp, ws);
    return hipErrorInvalidValue;
}

// Sum of the per-workgroup losses in a fixed order, added to the running bucket loss.
__global__ void __launch_bounds__(256)
k_loss_reduce(const double* __restrict__ partial, int64_t n, double* __restrict__ loss_sum) {
    __shared__ double sh[256];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 256) s += partial[i];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss_sum += sh[0];
}

hipError_t launch_loss_reduce(hipStream_t st, int64_t nwg, const Workspace& ws) {
    if (nwg <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_loss_reduce, dim3(1), dim3(256), 0, st, ws.loss_partial, nwg, ws.loss_sum);
    return hipGetLastError();
}

}  // namespace legend
