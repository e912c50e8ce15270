// Single-sweep batch computation for the common case: Eq. 1 loss, dim <= 128, at most 1024
// negatives per chunk (paper Sec. 2.1 stage 5, Sec. 6).  The general kernel reads the chunk's
// negatives twice because the row log-sum-exp must be known before any gradient.  Here the
// softmax numerators are taken against a reference known up front, the positive score f_e:
//     P_ek = exp(S_ek - f_e),   l_e = sum_k P_ek,   W_ek = P_ek / l_e,   loss_e = log l_e,
// so one sweep over the negatives yields the unnormalised G_Q = sum_k P_ek n_k, and the P
// blocks (64 x N values, the paper's "Intermediate Result 3") stay in the register file of the
// workgroup (256 accumulator registers per lane; one workgroup per compute unit) instead of
// going to global memory.  After the sweep the rows of Q are scaled by 1 / l_e and
// G_neg = P^T (Q / l) is formed straight from the stored blocks: the accumulator layout of a
// 32x32 MFMA block is exactly the A-operand layout of its transpose, so no LDS round trip.
// If some S_ek - f_e leaves [-60, 60] territory (overflow, or a row sum that underflows) the
// workgroup writes nothing and flags itself; the general two-sweep kernel then redoes it.
#include <type_traits>

#include "chunk_common.h"

namespace legend {

// compile-time loop: the body gets its index as an integral constant, so arrays indexed by it
// are scalarised into registers
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr int kFRow = 64, kFNeg = 64, kFWS = kFNeg + 4;
constexpr int kFastMaxTiles = 16;        // 1024 negatives

template <int NB, int SCORE, int DFIX>
__global__ void __launch_bounds__(kChunkThreads, 1)
k_chunk_fast(BatchGeom g, BucketParams bp, const int32_t* __restrict__ neg_ids, float* __restrict__ grad,
             double* __restrict__ loss_partial, uint32_t* __restrict__ redo) {
    constexpr int LPR = NB * 8;
    constexpr int RPS = kWave / LPR;
    constexpr int STEPS = 16 / RPS;
    constexpr int NBW = (2 * NB + 3) / 4;     // column blocks per wave in G_Q (as in the general kernel)

    extern __shared__ __align__(16) float smem[];
    const int d = DFIX ? DFIX : bp.dim;
    const int QS = chunk_row_stride(d);
    const int G_d = (d + 7) >> 3;
    const int tile_floats = kFRow * QS + 32 * NB;
    float* Qs = smem;
    float* Ns0 = Qs + tile_floats;
    float* Ns1 = Ns0 + tile_floats;
    float* Ws = Ns1 + tile_floats;              // [64][68]
    float* ref_s = Ws + kFRow * kFWS;           // [64] positive scores = softmax reference
    float* scale_s = ref_s + kFRow;             // [64] 1 / l_e
    float* logl_s = scale_s + kFRow;            // [64] log l_e
    float* rowloss_s = logl_s + kFRow;          // [64]
    uint32_t* flag_s = reinterpret_cast<uint32_t*>(rowloss_s + kFRow);   // [8]
    int32_t* ids_s = reinterpret_cast<int32_t*>(flag_s + 8);             // [kIdsLds]

    const int tid = threadIdx.x;
    const int w = tid >> 6;
    const int lane = tid & 63;
    const int i32 = lane & 31;
    const int kk = lane >> 5;

    int wg = blockIdx.x;
    const int t_row = wg % g.T;  wg /= g.T;
    const int c = wg % g.nchunks;
    const int si = wg / g.nchunks;
    const int side = g.side_id[si];
    const int chunk_rows = min(g.C, g.P - c * g.C);
    const int row0 = t_row * g.rows_tile;
    const int nrows = max(0, min(g.rows_tile, chunk_rows - row0));
    const int64_t e0 = (int64_t)c * g.C + row0;
    const int32_t* eb = bp.edges + (bp.batch_lo + e0) * 3;
    const float* Ex = side == 0 ? bp.E_src : bp.E_dst;
    const float* Ey = side == 0 ? bp.E_dst : bp.E_src;
    const float* En = Ey;
    const int xcol = side == 0 ? 0 : 2;
    const int ycol = 2 - xcol;
    const int N = g.N;
    const int32_t* my_negs = neg_ids + ((int64_t)si * g.nchunks + c) * N;
    const int64_t side_base = (int64_t)si * g.per_side;
    const int64_t neg_base = side_base + (int64_t)g.roles * g.P + ((int64_t)c * g.T + t_row) * N;
    const bool vec4 = (d & 3) == 0;
    const bool atomic = bp.atomic_mode != 0;

    for (int k = tid; k < N; k += kChunkThreads) ids_s[k] = my_negs[k];     // N <= 1024 here
    for (int idx = tid; idx < kFRow * (QS - d); idx += kChunkThreads) {
        int r = idx / (QS - d), cc = d + idx % (QS - d);
        Qs[r * QS + cc] = 0.f;
        Ns0[r * QS + cc] = 0.f;
        Ns1[r * QS + cc] = 0.f;
    }
    if (tid < 8) flag_s[tid] = 0;

    // ---- prologue: Q rows and positive scores; 4 threads per row ------------------------------
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
        if (ppart == 0) ref_s[prow] = partial;
    }
    __syncthreads();

    // ---- gather machinery (two tiles in flight, branch-free issue) ----------------------------
    float4 pf[2][STEPS];
    const int grow_lane = lane / LPR;
    const int gcol4 = lane % LPR;
    const int gc0 = gcol4 * 4;
    const int gcol_ld = gc0 < d ? gc0 : 0;
    typedef __attribute__((address_space(3))) const int32_t* lds_ids_t;
    auto gather_issue = [&](float4 (&buf)[STEPS], int n0) {
        int32_t idv[STEPS];
#pragma unroll
        for (int s = 0; s < STEPS; ++s) idv[s] = ((lds_ids_t)ids_s)[min(n0 + w * 16 + s * RPS + grow_lane, N - 1)];
        if (vec4) {
#pragma unroll
            for (int s = 0; s < STEPS; ++s) buf[s] = *reinterpret_cast<const float4*>(En + (int64_t)idv[s] * d + gcol_ld);
        } else {
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const float* p = En + (int64_t)idv[s] * d + gcol_ld;
                float4 v = make_float4(p[0], 0.f, 0.f, 0.f);
                if (gcol_ld + 1 < d) v.y = p[1];
                if (gcol_ld + 2 < d) v.z = p[2];
                if (gcol_ld + 3 < d) v.w = p[3];
                buf[s] = v;
            }
        }
    };
    auto gather_commit = [&](const float4 (&buf)[STEPS], float* Nt, int n0) {
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const int rt = w * 16 + s * RPS + grow_lane;
            float4 v = buf[s];
            if (n0 + rt >= N) v = make_float4(0.f, 0.f, 0.f, 0.f);
            float* dst = Nt + rt * QS + gc0;
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

    const int rbA = w & 1, cbA = w >> 1;
    auto score_block = [&](const float* Nt) -> f32x16 {
        f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        const float* qa = Qs + (rbA * 32 + i32) * QS + 4 * kk;
        const float* nb = Nt + (cbA * 32 + i32) * QS + 4 * kk;
        float4 a = lds4(qa), b = lds4(nb);
        for (int gi = 0; gi < G_d; ++gi) {
            float4 an = a, bn = b;
            if (gi + 1 < G_d) {
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
    auto acc_row = [&](int rb, int v) { return rb * 32 + 8 * (v >> 2) + 4 * kk + (v & 3); };

    const int ntiles = (N + kFNeg - 1) / kFNeg;
    const int rbG = w & 1;
    const int cb0 = w >> 1;
    const bool active = cb0 < NB;

    float ref_r[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) ref_r[v] = ref_s[acc_row(rbA, v)];
    float l_part[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) l_part[v] = 0.f;
    bool out_of_range = false;

    f32x16 P[kFastMaxTiles];                  // the chunk's softmax numerators, block by block
    f32x16 accB[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) accB[j][v] = 0.f;

    // ---- the sweep: scores, numerators, unnormalised G_Q ---------------------------------------
    gather_issue(pf[0], 0);
    if (ntiles > 1) gather_issue(pf[1], kFNeg);
    static_for<0, kFastMaxTiles>([&](auto T) {
        constexpr int t = decltype(T)::value;
        if (t < ntiles) {
            const int n0 = t * kFNeg;
            float* Nt = (t & 1) ? Ns1 : Ns0;
            gather_commit(pf[t & 1], Nt, n0);
            __syncthreads();                  // tile t visible; everyone is done with tile t-1 and its W
            if (t + 2 < ntiles) gather_issue(pf[t & 1], n0 + 2 * kFNeg);
            f32x16 acc = score_block(Nt);
            const bool col_ok = n0 + cbA * 32 + i32 < N;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = acc_row(rbA, v);
                const bool ok = col_ok && r < nrows;
                const float diff = acc[v] - ref_r[v];
                out_of_range |= ok && (diff > 60.f);
                const float p = ok ? fast_exp(diff) : 0.f;
                l_part[v] += p;
                acc[v] = p;
                Ws[r * kFWS + cbA * 32 + i32] = p;
            }
            P[t] = acc;
            __syncthreads();
            if (active) {
                const int G_n = (min(kFNeg, N - n0) + 7) >> 3;
                const float* wa = Ws + (rbG * 32 + i32) * kFWS + 4 * kk;
                const float* nb = Nt + (4 * kk) * QS + cb0 * 32 + i32;
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
        }
    });

    // ---- row sums: 64 partial holders per row (two waves x 32 lanes) ---------------------------
    __syncthreads();
    {
        const int pcol = cbA * 32 + i32;
#pragma unroll
        for (int v = 0; v < 16; ++v) Ws[acc_row(rbA, v) * kFWS + pcol] = l_part[v];
        if (__ballot(out_of_range) != 0ull && lane == 0) flag_s[w] = 1u;
    }
    __syncthreads();
    {
        const int srow = tid >> 2, sq = tid & 3;
        const float* wr = Ws + srow * kFWS + sq * 16;
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) sum += wr[j];
        sum += wave_shfl_xor(sum, 1);
        sum += wave_shfl_xor(sum, 2);
        if (sq == 0) {
            const bool live = srow < nrows;
            // a row sum that is tiny or not finite means the reference was a poor one for this row
            if (live && !(sum > 1e-30f && sum < 1e30f)) flag_s[4] = 1u;
            scale_s[srow] = live ? 1.f / sum : 0.f;
            logl_s[srow] = live ? logf(sum) : 0.f;
        }
    }
    __syncthreads();
    const bool bad = (flag_s[0] | flag_s[1] | flag_s[2] | flag_s[3] | flag_s[4]) != 0u;
    if (tid == 0) redo[blockIdx.x] = bad ? 1u : 0u;
    if (bad) return;                          // uniform: nothing has been written yet

    // ---- Q <- Q / l (row-wise), so that G_neg = P^T Q' ------------------------------------------
    if (prow < nrows) {
        const float sc = scale_s[prow];
        for (int k = ppart; k < d; k += 4) Qs[prow * QS + k] *= sc;
    }
    __syncthreads();

    // ---- G_neg, tile by tile, straight from the stored blocks -----------------------------------
    // Wave (rbA, cbA) holds P for rows of block rbA and negatives of block cbA: its accumulator
    // layout is the A operand of P^T for those 32 rows, so it computes the contribution of its
    // rows to all column blocks; the two row blocks are added in the staging tile.
    const int rows_in_block = max(0, min(32, nrows - rbA * 32));
    const int G_r = (rows_in_block + 7) >> 3;
    static_for<0, kFastMaxTiles>([&](auto T) {
        constexpr int t = decltype(T)::value;
        if (t < ntiles) {
            const int n0 = t * kFNeg;
            float* St = (t & 1) ? Ns1 : Ns0;  // staging tile
            f32x16 accC[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) accC[j][v] = 0.f;
            const float* qb = Qs + (rbA * 32 + 4 * kk) * QS + i32;
#pragma unroll
            for (int gi = 0; gi < 4; ++gi) {
                if (gi < G_r) {
                    float b[NB][4];
#pragma unroll
                    for (int j = 0; j < NB; ++j)
#pragma unroll
                        for (int s = 0; s < 4; ++s) b[j][s] = qb[(8 * gi + s) * QS + 32 * j];
#pragma unroll
                    for (int j = 0; j < NB; ++j)
#pragma unroll
                        for (int s = 0; s < 4; ++s) accC[j] = mfma32(P[t][4 * gi + s], b[j][s], accC[j]);
                }
            }
            // staging: row block 0 writes, row block 1 adds
            if (rbA == 0) {
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int col = j * 32 + i32;
                    if (col < d) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) St[(cbA * 32 + 8 * (v >> 2) + 4 * kk + (v & 3)) * QS + col] = accC[j][v];
                    }
                }
            }
            __syncthreads();
            if (rbA == 1) {
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int col = j * 32 + i32;
                    if (col < d) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) St[(cbA * 32 + 8 * (v >> 2) + 4 * kk + (v & 3)) * QS + col] += accC[j][v];
                    }
                }
            }
            __syncthreads();
            if (atomic) {
                float* Gn = side == 0 ? bp.G_dst : bp.G_src;
#pragma unroll
                for (int s = 0; s < STEPS; ++s) {
                    const int rt = w * 16 + s * RPS + grow_lane;
                    const int neg = n0 + rt;
                    if (neg < N && gc0 < d) {
                        const float* src = St + rt * QS + gc0;
                        float* dst = Gn + (int64_t)ids_s[neg] * d + gc0;
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
                        const float* src = St + rt * QS + gc0;
                        float* dst = grad + (neg_base + neg) * d + gc0;
                        if (vec4) {
                            *reinterpret_cast<float4*>(dst) = lds4(src);
                        } else {
                            dst[0] = src[0];
                            if (gc0 + 1 < d) dst[1] = src[1];
                            if (gc0 + 2 < d) dst[2] = src[2];
                            if (gc0 + 3 < d) dst[3] = src[3];
                        }
                    }
                }
            }
            // the other staging tile is used next; this one is rewritten two barriers from now
        }
    });
    __syncthreads();

    // ---- epilogue: G_Q (unnormalised) to LDS, chain rule, gradient rows of the positives --------
    float* Gs = Ns0;
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
    __syncthreads();
    auto emit = [&](float* p, float v) {
        if (atomic) unsafeAtomicAdd(p, v);
        else *p = v;
    };
    {
        float row_loss = 0.f;
        if (prow < nrows) {
            const float sc = scale_s[prow];
            row_loss = logl_s[prow];          // lse - f with the positive score as reference
            const float a = -1.f;
            const float* x = Ex + (int64_t)eb[prow * 3 + xcol] * d;
            const float* y = Ey + (int64_t)eb[prow * 3 + ycol] * d;
            const float* r = SCORE == LEGEND_SCORE_DOT ? x : bp.E_rel + (int64_t)eb[prow * 3 + 1] * d;
            const int64_t e = e0 + prow;
            float* gx = grad + (side_base + (side == 0 ? 0 : g.P) + e) * d;
            float* gy = grad + (side_base + (side == 0 ? g.P : 0) + e) * d;
            float* gr = grad + (side_base + 2 * (int64_t)g.P + e) * d;
            if (atomic) {
                gx = (side == 0 ? bp.G_src : bp.G_dst) + (int64_t)eb[prow * 3 + xcol] * d;
                gy = (side == 0 ? bp.G_dst : bp.G_src) + (int64_t)eb[prow * 3 + ycol] * d;
                gr = bp.G_rel + (int64_t)eb[prow * 3 + 1] * d;
            }
            const float* gq = Gs + prow * QS;
            if (SCORE == LEGEND_SCORE_COMPLEX) {
                const int h = d >> 1;
                for (int k = ppart; k < h; k += 4) {
                    float xr = x[k], xi = x[k + h], rr = r[k], ri = r[k + h];
                    float qr, qi;
                    if (side == 0) { qr = xr * rr - xi * ri; qi = xr * ri + xi * rr; }
                    else           { qr = rr * xr + ri * xi; qi = rr * xi - ri * xr; }
                    float gre = gq[k] * sc + a * y[k], gim = gq[k + h] * sc + a * y[k + h];
                    emit(gy + k, a * qr);
                    emit(gy + k + h, a * qi);
                    if (side == 0) {
                        emit(gx + k, rr * gre + ri * gim);      emit(gx + k + h, rr * gim - ri * gre);
                        emit(gr + k, xr * gre + xi * gim);      emit(gr + k + h, xr * gim - xi * gre);
                    } else {
                        emit(gx + k, rr * gre - ri * gim);      emit(gx + k + h, rr * gim + ri * gre);
                        emit(gr + k, gre * xr + gim * xi);      emit(gr + k + h, gre * xi - gim * xr);
                    }
                }
            } else {
                for (int k = ppart; k < d; k += 4) {
                    const float q = SCORE == LEGEND_SCORE_DOT ? x[k] : x[k] * r[k];
                    const float gv = gq[k] * sc + a * y[k];
                    emit(gy + k, a * q);
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
        for (int r = 0; r < kFRow; ++r) s += (double)rowloss_s[r];
        loss_partial[blockIdx.x] = s;
    }
}

static size_t fast_lds_bytes(int d, int nb) {
    const int QS = chunk_row_stride(d);
    size_t floats = 3 * ((size_t)kFRow * QS + 32 * nb) + (size_t)kFRow * kFWS + 4 * kFRow + 8 + kIdsLds;
    return floats * sizeof(float);
}

// Built only for the dimensions of the paper's workloads (the fully unrolled sweep is expensive
// to compile); every other shape takes the general kernel.
bool chunk_fast_applies(const BatchGeom& g, const BucketParams& bp) {
    if (bp.loss != LEGEND_LOSS_SOFTMAX || g.N > kFastMaxTiles * kFNeg || g.N > kIdsLds) return false;
    return bp.dim == 100 || (bp.dim == 32 && bp.score == LEGEND_SCORE_DOT);
}

template <int NB, int SC, int DFIX>
static hipError_t launch_fast_one(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    dim3 grid((unsigned)(g.sides * g.nchunks * g.T)), block(kChunkThreads);
    const size_t lds = fast_lds_bytes(bp.dim, NB);
    static size_t lds_allowed = 0;
    if (lds > lds_allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_chunk_fast<NB, SC, DFIX>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        lds_allowed = lds;
    }
    hipLaunchKernelGGL((k_chunk_fast<NB, SC, DFIX>), grid, block, lds, st, g, bp, ws.neg_ids, ws.grad,
                       ws.loss_partial, ws.redo);
    return hipGetLastError();
}

hipError_t launch_chunks_fast(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    if (bp.dim == 100) {
        if (bp.score == LEGEND_SCORE_DOT) return launch_fast_one<4, LEGEND_SCORE_DOT, 100>(st, g, bp, ws);
        if (bp.score == LEGEND_SCORE_DISTMULT) return launch_fast_one<4, LEGEND_SCORE_DISTMULT, 100>(st, g, bp, ws);
        return launch_fast_one<4, LEGEND_SCORE_COMPLEX, 100>(st, g, bp, ws);
    }
    if (bp.dim == 32 && bp.score == LEGEND_SCORE_DOT) return launch_fast_one<1, LEGEND_SCORE_DOT, 32>(st, g, bp, ws);
    return hipErrorInvalidValue;
}

}  // namespace legend
