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
#include <type_traits>

#include "chunk_common.h"

namespace legend {

constexpr int kRowTile = 64;    // positives per workgroup (padded)
constexpr int kNegTile = 64;    // negatives per LDS tile
constexpr int kWS = kNegTile + 4;   // row stride of the W tile: a multiple of 4 that is 4 mod 8

int row_tiles_for(int chunk_size, int dim) {
    const int tile = dim > kNarrowMaxDim ? kWideRowTile : kRowTile;
    return (chunk_size + tile - 1) / tile;
}
int rows_per_tile_for(int chunk_size, int dim) {
    int t = row_tiles_for(chunk_size, dim);
    return (chunk_size + t - 1) / t;
}
int max_dim_supported() { return kWideMaxDim; }
bool dim_supported(int dim) { return dim >= 1 && dim <= kWideMaxDim; }

// NB: number of 32-wide column blocks covering the embedding dimension (dim <= 32 * NB).
// DFIX: the embedding dimension when it is known at compile time (strides, trip counts and
// the float4 path fold to constants), or 0 to take it from the arguments.
template <int NB, int SCORE, int LOSS, int DFIX>
__global__ void __launch_bounds__(kChunkThreads, 2)     // two waves per SIMD: two workgroups share a compute unit
k_chunk(BatchGeom g, BucketParams bp, const int32_t* __restrict__ neg_ids, float* __restrict__ grad,
        double* __restrict__ loss_partial, const uint32_t* __restrict__ only_if) {
    // redo mode: only the workgroups the single-sweep kernel flagged have anything to do
    if (only_if && only_if[blockIdx.x] == 0u) return;
    constexpr int LPR = NB * 8;             // lanes that cooperate on one gathered row (float4 each)
    constexpr int RPS = kWave / LPR;        // rows a wave gathers per step
    constexpr int STEPS = 16 / RPS;         // each wave gathers 16 of the 64 tile rows
    constexpr int NBW = (2 * NB + 3) / 4;   // 32x32 output blocks per wave in the gradient products

    extern __shared__ __align__(16) float smem[];
    const int d = DFIX ? DFIX : bp.dim;
    const int QS = chunk_row_stride(d);
    const int G_d = (d + 7) >> 3;           // contraction groups over the embedding dimension
    const int tile_floats = kRowTile * QS + 32 * NB;
    float* Qs = smem;                       // [64][QS]  Q rows of this workgroup
    float* Ns = Qs + tile_floats;           // [64][QS]  current negative tile (later: G_Q)
    float* Ws = Ns + tile_floats;           // [64][68]  W of the current tile (also reduction scratch)
    float* pos_s = Ws + kRowTile * kWS;     // [64]
    float* lse_s = pos_s + kRowTile;        // [64]
    float* rowloss_s = lse_s + kRowTile;    // [64]
    int32_t* ids_s = reinterpret_cast<int32_t*>(rowloss_s + kRowTile);   // [kIdsLds]

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

    // ---- negative ids of the chunk, and zero pad columns [d, QS) of both row tiles -----------
    for (int k = tid; k < min(N, kIdsLds); k += kChunkThreads) ids_s[k] = my_negs[k];
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
    __syncthreads();                          // ids_s, Qs, pos_s complete

    // ---- negative tile gather: rows travel through registers (up to three tiles in flight) and
    // are committed to LDS when the previous tile is done.  Buffer indices are compile-time
    // (the tile loops are unrolled by the number of buffers) so the buffers stay in registers.
    float4 pf[3][STEPS];
    const int grow_lane = lane / LPR;         // row within a step
    const int gcol4 = lane % LPR;             // float4 column
    const int gc0 = gcol4 * 4;
    // Straight-line code on purpose: rows past the end of the chunk's negatives and lanes past
    // the end of a row load some valid address and are zeroed when the tile is committed, so
    // that all loads of a tile are issued back to back and nothing waits on them here.
    const bool ids_in_lds = N <= kIdsLds;     // uniform: all ids of the chunk sit in LDS
    const int gcol_ld = gc0 < d ? gc0 : 0;
    auto gather_issue = [&](auto BUF, int n0) {
        constexpr int B = decltype(BUF)::value;
        int32_t idv[STEPS];
        if (ids_in_lds) {
            // explicit LDS address space: keeps these reads apart from the global path below
            typedef __attribute__((address_space(3))) const int32_t* lds_ids_t;
            lds_ids_t ids_l = (lds_ids_t)ids_s;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) idv[s] = ids_l[min(n0 + w * 16 + s * RPS + grow_lane, N - 1)];
        } else {
#pragma unroll
            for (int s = 0; s < STEPS; ++s) idv[s] = my_negs[min(n0 + w * 16 + s * RPS + grow_lane, N - 1)];
        }
        if (vec4) {
#pragma unroll
            for (int s = 0; s < STEPS; ++s)
                pf[B][s] = *reinterpret_cast<const float4*>(En + (int64_t)idv[s] * d + gcol_ld);
        } else if ((d & 1) == 0) {
            // an even dimension that is no multiple of four: rows are 8-byte aligned, two 64-bit loads
            const bool second = gcol_ld + 2 < d;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const float* p = En + (int64_t)idv[s] * d + gcol_ld;
                const float2 a = *reinterpret_cast<const float2*>(p);
                const float2 b = *reinterpret_cast<const float2*>(second ? p + 2 : p);
                pf[B][s] = make_float4(a.x, a.y, second ? b.x : 0.f, second ? b.y : 0.f);
            }
        } else {
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const float* p = En + (int64_t)idv[s] * d + gcol_ld;
                float4 v = make_float4(p[0], 0.f, 0.f, 0.f);
                if (gcol_ld + 1 < d) v.y = p[1];
                if (gcol_ld + 2 < d) v.z = p[2];
                if (gcol_ld + 3 < d) v.w = p[3];
                pf[B][s] = v;
            }
        }
    };
    auto gather_commit = [&](auto BUF, int n0) {
        constexpr int B = decltype(BUF)::value;
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const int rt = w * 16 + s * RPS + grow_lane;
            const bool row_ok = n0 + rt < N;
            float4 v = pf[B][s];
            if (!row_ok) v = make_float4(0.f, 0.f, 0.f, 0.f);
            float* dst = Ns + rt * QS + gc0;
            if (vec4) {
                if (gc0 < d) *reinterpret_cast<float4*>(dst) = v;
            } else {
                if (gc0 < d) dst[0] = v.x;
                if (gc0 + 1 < d) dst[1] = v.y;
                if (gc0 + 2 < d) dst[2] = v.z;
                if (gc0 + 3 < d) dst[3] = v.w;
            }
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;

    // ---- S block of this wave: rows rbA*32.., negatives cbA*32.. of the current tile --------
    const int rbA = w & 1, cbA = w >> 1;
    auto score_block = [&]() -> f32x16 {
        f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        const float* qa = Qs + (rbA * 32 + i32) * QS + 4 * kk;
        const float* nb = Ns + (cbA * 32 + i32) * QS + 4 * kk;
        float4 a = lds4(qa), b = lds4(nb);
        for (int gi = 0; gi < G_d; ++gi) {
            float4 an = a, bn = b;
            if (gi + 1 < G_d) {               // operands of the next group travel while this group multiplies
                an = lds4(qa + 8 * (gi + 1));
                bn = lds4(nb + 8 * (gi + 1));
            }
            __builtin_amdgcn_sched_barrier(0);
            acc = mfma32(a.x, b.x, acc);
            acc = mfma32(a.y, b.y, acc);
            acc = mfma32(a.z, b.z, acc);
            acc = mfma32(a.w, b.w, acc);
            __builtin_amdgcn_sched_barrier(0);
            a = an;
            b = bn;
        }
        return acc;
    };
    // row of accumulator element v of a 32x32 block with row block rb
    auto acc_row = [&](int rb, int v) { return rb * 32 + 8 * (v >> 2) + 4 * kk + (v & 3); };

    const int ntiles = (N + kNegTile - 1) / kNegTile;
    const int srow = tid >> 2;                // 4 threads per row for the row-wise reductions
    const int sq = tid & 3;
    float neg_loss = 0.f;                     // logistic / margin: this lane's share of the negatives' loss terms
    float cnt_l[LOSS == LEGEND_LOSS_MARGIN ? 16 : 1];         // margin: violating negatives per row among this lane's columns
#pragma unroll
    for (int v = 0; v < (LOSS == LEGEND_LOSS_MARGIN ? 16 : 1); ++v) cnt_l[v] = 0.f;

    if (LOSS == LEGEND_LOSS_SOFTMAX) {
        // ---- sweep 1: running max and sum of exp, per lane over its own columns -------------
        // Each lane keeps, per row, a reference score m and sum of exp(S - m) over the columns it
        // has seen.  The reference only moves when a score exceeds it by more than 16 (the sum
        // then stays far inside the fp32 range), so the common case costs one exp per score.
        // This sweep has little arithmetic per gathered byte, so three tiles are kept in flight.
        float m_l[16], s_l[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) { m_l[v] = -INFINITY; s_l[v] = 0.f; }
        bool seeded = false;
        auto sweep1_tile = [&](auto BUF, auto NEXT, int tile) {
            if (tile >= ntiles) return;
            const int n0 = tile * kNegTile;
            gather_commit(BUF, n0);
            __syncthreads();
            if (tile + 2 < ntiles) gather_issue(NEXT, n0 + 2 * kNegTile);
            f32x16 acc = score_block();
            if (n0 + cbA * 32 + i32 < N) {
                if (!seeded) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) { m_l[v] = acc[v]; s_l[v] = 1.f; }
                    seeded = true;
                } else {
                    float tmax = acc[0] - m_l[0];
#pragma unroll
                    for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, acc[v] - m_l[v]);
                    if (tmax <= 16.f) {       // common case, no branch per score
#pragma unroll
                        for (int v = 0; v < 16; ++v) s_l[v] += fast_exp(acc[v] - m_l[v]);
                    } else {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const float tdiff = acc[v] - m_l[v];
                            if (tdiff > 16.f) {
                                s_l[v] = fmaf(s_l[v], fast_exp(-tdiff), 1.f);
                                m_l[v] = acc[v];
                            } else {
                                s_l[v] += fast_exp(tdiff);
                            }
                        }
                    }
                }
            }
            __syncthreads();
        };
        gather_issue(I0{}, 0);
        if (ntiles > 1) gather_issue(I1{}, kNegTile);
        for (int tile = 0; tile < ntiles; tile += 3) {
            sweep1_tile(I0{}, I2{}, tile);
            sweep1_tile(I1{}, I0{}, tile + 1);
            sweep1_tile(I2{}, I1{}, tile + 2);
        }
        // combine the 64 per-lane partials of every row (two waves x 32 lanes): max, then sum
        const int pcol = cbA * 32 + i32;
#pragma unroll
        for (int v = 0; v < 16; ++v) Ws[acc_row(rbA, v) * kWS + pcol] = m_l[v];
        __syncthreads();
        {
            const float* wr = Ws + srow * kWS + sq * 16;
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < 16; ++j) mx = fmaxf(mx, wr[j]);
            mx = fmaxf(mx, wave_shfl_xor(mx, 1));
            mx = fmaxf(mx, wave_shfl_xor(mx, 2));
            if (sq == 0) lse_s[srow] = mx;
        }
        __syncthreads();
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = acc_row(rbA, v);
            Ws[r * kWS + pcol] = s_l[v] * expf(m_l[v] - lse_s[r]);   // a lane without columns has s_l = 0
        }
        __syncthreads();
        {
            const float* wr = Ws + srow * kWS + sq * 16;
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < 16; ++j) sum += wr[j];
            sum += wave_shfl_xor(sum, 1);
            sum += wave_shfl_xor(sum, 2);
            const float mx = lse_s[srow];
            __syncthreads();                  // every thread has read the row maxima
            if (sq == 0) {
                float lse = mx + logf(sum);
                if (bp.softmax_with_pos) {    // the positive score joins the log-sum-exp
                    const float f = pos_s[srow];
                    // x = lse over the negatives - f is kept: the loss term is softplus(x) and dL/df is
                    // -sigmoid(x), both accurate where the positive dominates (lse' - f itself cancels there)
                    rowloss_s[srow] = lse - f;
                    const float hi = fmaxf(lse, f), lo = fminf(lse, f);
                    lse = hi + log1pf(expf(lo - hi));
                }
                lse_s[srow] = lse;
            }
        }
        __syncthreads();
    }

    // ---- sweep 2: gradients ----------------------------------------------------------------
    f32x16 accB[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) accB[j][v] = 0.f;
    const int rbG = w & 1;
    const int cb0 = w >> 1;                   // first column block of this wave; the j-th is cb0 + 2j
    const bool active = cb0 < NB;             // NB = 1: only two waves have an output block
    const int G_rows = (nrows + 7) >> 3;
    const float wneg = bp.neg_weight;

    auto sweep2_tile = [&](auto BUF, int tile) {
        if (tile >= ntiles) return;
        const int n0 = tile * kNegTile;
        gather_commit(BUF, n0);
        __syncthreads();
        if (tile + 2 < ntiles) gather_issue(BUF, n0 + 2 * kNegTile);   // this buffer is free again
        {
            f32x16 acc = score_block();
            const bool col_ok = n0 + cbA * 32 + i32 < N;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = acc_row(rbA, v);
                float wv = 0.f;
                if (col_ok && r < nrows) {
                    if (LOSS == LEGEND_LOSS_SOFTMAX) {
                        wv = fast_exp(acc[v] - lse_s[r]);
                    } else if (LOSS == LEGEND_LOSS_MARGIN) {
                        // pairwise hinge max(0, margin - f + S): dL/dS is 1 for a negative less than the margin
                        // below the positive (0 on the hinge itself)
                        const float sh = (bp.margin - pos_s[r]) + acc[v];
                        wv = sh > 0.f ? 1.f : 0.f;
                        neg_loss += fmaxf(sh, 0.f);
                        cnt_l[LOSS == LEGEND_LOSS_MARGIN ? v : 0] += wv;
                    } else {
                        wv = wneg * sigmoidf(acc[v]);
                        neg_loss += wneg * softplusf(acc[v]);
                    }
                }
                Ws[r * kWS + cbA * 32 + i32] = wv;
            }
        }
        __syncthreads();
        f32x16 accC[NBW];
#pragma unroll
        for (int j = 0; j < NBW; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) accC[j][v] = 0.f;
        if (active) {
            const int G_n = (min(kNegTile, N - n0) + 7) >> 3;
            // G_Q += W * Neg : contraction over the negatives of the tile
            {
                const float* wa = Ws + (rbG * 32 + i32) * kWS + 4 * kk;
                const float* nb = Ns + (4 * kk) * QS + cb0 * 32 + i32;
                for (int gi = 0; gi < G_n; ++gi) {
                    const float4 a = lds4(wa + 8 * gi);
                    const float* nbg = nb + 8 * gi * QS;
                    float b[NBW][4];
#pragma unroll
                    for (int j = 0; j < NBW; ++j)
#pragma unroll
                        for (int s = 0; s < 4; ++s) b[j][s] = nbg[s * QS + 64 * j];
#pragma unroll
                    for (int j = 0; j < NBW; ++j) {
                        accB[j] = mfma32(a.x, b[j][0], accB[j]);
                        accB[j] = mfma32(a.y, b[j][1], accB[j]);
                        accB[j] = mfma32(a.z, b[j][2], accB[j]);
                        accB[j] = mfma32(a.w, b[j][3], accB[j]);
                    }
                }
            }
            // G_neg = W^T * Q : contraction over the positives
            {
                const float* wa = Ws + (4 * kk) * kWS + rbG * 32 + i32;
                const float* qb = Qs + (4 * kk) * QS + cb0 * 32 + i32;
                for (int gi = 0; gi < G_rows; ++gi) {
                    const float* wag = wa + 8 * gi * kWS;
                    const float* qbg = qb + 8 * gi * QS;
                    float a[4], b[NBW][4];
#pragma unroll
                    for (int s = 0; s < 4; ++s) a[s] = wag[s * kWS];
#pragma unroll
                    for (int j = 0; j < NBW; ++j)
#pragma unroll
                        for (int s = 0; s < 4; ++s) b[j][s] = qbg[s * QS + 64 * j];
#pragma unroll
                    for (int j = 0; j < NBW; ++j)
#pragma unroll
                        for (int s = 0; s < 4; ++s) accC[j] = mfma32(a[s], b[j][s], accC[j]);
                }
            }
        }
        __syncthreads();                      // the negative tile is not read any more
        // G_neg goes through the tile buffer so that whole gradient rows leave as 16-byte stores
        if (active) {
#pragma unroll
            for (int j = 0; j < NBW; ++j) {
                const int col = (cb0 + 2 * j) * 32 + i32;
                if (col < d) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) Ns[acc_row(rbG, v) * QS + col] = accC[j][v];
                }
            }
        }
        __syncthreads();
        if (bp.atomic_mode) {
            // atomic mode: add the rows to the accumulator of the negatives' table
            float* Gn = side == 0 ? bp.G_dst : bp.G_src;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const int rt = w * 16 + s * RPS + grow_lane;
                const int neg = n0 + rt;
                if (neg < N && gc0 < d) {
                    const int32_t id = neg < kIdsLds ? ids_s[neg] : my_negs[neg];
                    const float* src = Ns + rt * QS + gc0;
                    float* dst = Gn + (int64_t)id * d + gc0;
                    unsafeAtomicAdd(dst, src[0]);
                    if (gc0 + 1 < d) unsafeAtomicAdd(dst + 1, src[1]);
                    if (gc0 + 2 < d) unsafeAtomicAdd(dst + 2, src[2]);
                    if (gc0 + 3 < d) unsafeAtomicAdd(dst + 3, src[3]);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const int rt = w * 16 + s * RPS + grow_lane;
                const int neg = n0 + rt;
                if (neg < N && gc0 < d) {
                    const float* src = Ns + rt * QS + gc0;
                    float* dst = grad + (neg_base + neg) * d + gc0;
                    if (vec4) {
                        *reinterpret_cast<float4*>(dst) = lds4(src);
                    } else if ((d & 1) == 0) {
                        const float4 v = lds4(src);
                        *reinterpret_cast<float2*>(dst) = make_float2(v.x, v.y);
                        if (gc0 + 2 < d) *reinterpret_cast<float2*>(dst + 2) = make_float2(v.z, v.w);
                    } else {
                        dst[0] = src[0];
                        if (gc0 + 1 < d) dst[1] = src[1];
                        if (gc0 + 2 < d) dst[2] = src[2];
                        if (gc0 + 3 < d) dst[3] = src[3];
                    }
                }
            }
        }
        __syncthreads();                      // staged rows are read; the next tile may be committed
    };
    gather_issue(I0{}, 0);
    if (ntiles > 1) gather_issue(I1{}, kNegTile);
    for (int tile = 0; tile < ntiles; tile += 2) {
        sweep2_tile(I0{}, tile);
        sweep2_tile(I1{}, tile + 1);
    }

    // ---- epilogue: G_Q to LDS, chain rule, gradient rows of the positives -------------------
    float* Gs = Ns;
    const bool atomic = bp.atomic_mode != 0;
    auto emit = [&](float* p, float v) {
        if (atomic) unsafeAtomicAdd(p, v);
        else *p = v;
    };
    if (active) {
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
            const int col = (cb0 + 2 * j) * 32 + i32;
            if (col < d) {
#pragma unroll
                for (int v = 0; v < 16; ++v) Gs[acc_row(rbG, v) * QS + col] = accB[j][v];
            }
        }
    }
    if (LOSS == LEGEND_LOSS_MARGIN) {
        // dL/df of a row is minus the number of its violating negatives: combine the 64 per-lane counts of
        // every row (two waves x 32 lanes); small integers, exact in any order
        __syncthreads();                      // the last tile's W has been consumed
        const int pcol = cbA * 32 + i32;
#pragma unroll
        for (int v = 0; v < 16; ++v) Ws[acc_row(rbA, v) * kWS + pcol] = cnt_l[LOSS == LEGEND_LOSS_MARGIN ? v : 0];
        __syncthreads();
        const float* wr = Ws + srow * kWS + sq * 16;
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) sum += wr[j];
        sum += wave_shfl_xor(sum, 1);
        sum += wave_shfl_xor(sum, 2);
        if (sq == 0) rowloss_s[srow] = sum;
    }
    if (LOSS == LEGEND_LOSS_LOGISTIC || LOSS == LEGEND_LOSS_MARGIN) {
        // workgroup total of the negative terms: lanes -> wave -> LDS
        for (int off = kWave / 2; off > 0; off >>= 1) neg_loss += __shfl_down(neg_loss, off, kWave);
        if (lane == 0) lse_s[w] = neg_loss;
    }
    __syncthreads();
    {
        float row_loss = 0.f;
        if (prow < nrows) {
            const float f = pos_s[prow];
            float a;
            if (LOSS == LEGEND_LOSS_SOFTMAX) {
                if (bp.softmax_with_pos) {
                    const float x = rowloss_s[prow];          // read by the row's four lanes before one of them reuses the slot
                    row_loss = softplusf(x);
                    a = -sigmoidf(x);
                } else {
                    row_loss = lse_s[prow] - f;
                    a = -1.f;
                }
            }
            else if (LOSS == LEGEND_LOSS_MARGIN) { a = -rowloss_s[prow]; row_loss = 0.f; }   // read by the row's four lanes before the slot is reused
            else { a = -sigmoidf(-f); row_loss = softplusf(-f); }
            const float* x = Ex + (int64_t)eb[prow * 3 + xcol] * d;
            const float* y = Ey + (int64_t)eb[prow * 3 + ycol] * d;
            const float* r = SCORE == LEGEND_SCORE_DOT ? x : bp.E_rel + (int64_t)eb[prow * 3 + 1] * d;
            const int64_t e = e0 + prow;
            float* gx = grad + (side_base + (side == 0 ? 0 : g.P) + e) * d;        // source rows first
            float* gy = grad + (side_base + (side == 0 ? g.P : 0) + e) * d;
            float* gr = grad + (side_base + 2 * (int64_t)g.P + e) * d;
            if (atomic) {                     // straight into the per-table gradient accumulators
                gx = (side == 0 ? bp.G_src : bp.G_dst) + (int64_t)eb[prow * 3 + xcol] * d;
                gy = (side == 0 ? bp.G_dst : bp.G_src) + (int64_t)eb[prow * 3 + ycol] * d;
                gr = bp.G_rel + (int64_t)eb[prow * 3 + 1] * d;
            }
            const float* gq = Gs + prow * QS;
            const float* q = Qs + prow * QS;
            if (SCORE == LEGEND_SCORE_COMPLEX) {
                const int h = d >> 1;
                for (int k = ppart; k < h; k += 4) {
                    float gre = gq[k] + a * y[k], gim = gq[k + h] + a * y[k + h];
                    float xr = x[k], xi = x[k + h], rr = r[k], ri = r[k + h];
                    emit(gy + k, a * q[k]);
                    emit(gy + k + h, a * q[k + h]);
                    if (side == 0) {
                        emit(gx + k, rr * gre + ri * gim);      emit(gx + k + h, rr * gim - ri * gre);   // conj(r) g
                        emit(gr + k, xr * gre + xi * gim);      emit(gr + k + h, xr * gim - xi * gre);   // conj(x) g
                    } else {
                        emit(gx + k, rr * gre - ri * gim);      emit(gx + k + h, rr * gim + ri * gre);   // r g
                        emit(gr + k, gre * xr + gim * xi);      emit(gr + k + h, gre * xi - gim * xr);   // conj(g) x
                    }
                }
            } else {
                for (int k = ppart; k < d; k += 4) {
                    float gv = gq[k] + a * y[k];
                    emit(gy + k, a * q[k]);
                    if (SCORE == LEGEND_SCORE_DOT) {
                        emit(gx + k, gv);
                    } else {
                        emit(gx + k, r[k] * gv);
                        emit(gr + k, x[k] * gv);
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
        if (LOSS == LEGEND_LOSS_LOGISTIC || LOSS == LEGEND_LOSS_MARGIN)
            for (int ww = 0; ww < kChunkThreads / kWave; ++ww) s += (double)lse_s[ww];
        loss_partial[blockIdx.x] = s;
    }
}

static size_t chunk_lds_bytes(int d, int nb) {
    int QS = chunk_row_stride(d);
    size_t floats = 2 * ((size_t)kRowTile * QS + 32 * nb) + (size_t)kRowTile * kWS + 3 * kRowTile + kIdsLds;
    return floats * sizeof(float);
}

template <int NB, int DFIX>
static hipError_t launch_chunks_nb(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws,
                                   const uint32_t* only_if) {
    dim3 grid((unsigned)(g.sides * g.nchunks * g.T)), block(kChunkThreads);
    size_t lds = chunk_lds_bytes(bp.dim, NB);
#define LEGEND_CHUNK_CASE(SC, LO)                                                                              \
    if (bp.score == SC && bp.loss == LO) {                                                                     \
        static size_t lds_allowed = 0; /* dynamic LDS above 64 KB has to be requested per kernel */            \
        if (lds > lds_allowed) {                                                                               \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_chunk<NB, SC, LO, DFIX>),      \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
            if (e != hipSuccess) return e;                                                                     \
            lds_allowed = lds;                                                                                 \
        }                                                                                                      \
        hipLaunchKernelGGL((k_chunk<NB, SC, LO, DFIX>), grid, block, lds, st, g, bp, ws.neg_ids, ws.grad,      \
                           ws.loss_partial, only_if);                                                          \
        return hipGetLastError();                                                                              \
    }
    LEGEND_CHUNK_CASE(LEGEND_SCORE_DOT, LEGEND_LOSS_SOFTMAX)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_DOT, LEGEND_LOSS_LOGISTIC)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_DISTMULT, LEGEND_LOSS_SOFTMAX)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_DISTMULT, LEGEND_LOSS_LOGISTIC)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_COMPLEX, LEGEND_LOSS_SOFTMAX)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_COMPLEX, LEGEND_LOSS_LOGISTIC)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_DOT, LEGEND_LOSS_MARGIN)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_DISTMULT, LEGEND_LOSS_MARGIN)
    LEGEND_CHUNK_CASE(LEGEND_SCORE_COMPLEX, LEGEND_LOSS_MARGIN)
#undef LEGEND_CHUNK_CASE
    return hipErrorInvalidValue;
}

bool chunks_use_single_sweep(const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    return g.P > 0 && bp.score != LEGEND_SCORE_TRANSE_L1 && chunk_fast_applies(g, bp) && !ws.no_fast_path;
}

// redo = false: the batch computation proper.  redo = true (only after a single-sweep launch):
// the two-sweep kernel over the workgroups the single-sweep kernel flagged as out of range.
hipError_t launch_chunks(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws, bool redo) {
    if (g.P <= 0) return hipSuccess;
    const bool single = chunks_use_single_sweep(g, bp, ws);
    if (redo && !single) return hipSuccess;
    if (!redo && single) return launch_chunks_fast(st, g, bp, ws);
    if (bp.score == LEGEND_SCORE_TRANSE_L1) return launch_chunks_trans(st, g, bp, ws);
    const uint32_t* only_if = redo ? ws.redo : nullptr;
    // the dimensions of the paper's workloads get kernels with the dimension folded in
    if (bp.dim == 100) return launch_chunks_nb<4, 100>(st, g, bp, ws, only_if);
    if (bp.dim == 32) return launch_chunks_nb<1, 32>(st, g, bp, ws, only_if);
    if (bp.dim <= 32) return launch_chunks_nb<1, 0>(st, g, bp, ws, only_if);
    if (bp.dim <= 64) return launch_chunks_nb<2, 0>(st, g, bp, ws, only_if);
    if (bp.dim <= 128) return launch_chunks_nb<4, 0>(st, g, bp, ws, only_if);
    return launch_chunks_gemm(st, g, bp, ws);
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
