// Batch computation for embedding dimensions 129..512 (multiples of 4), e.g. the d = 400
// knowledge-graph configuration.  Same mathematics and the same two sweeps as the narrow
// kernel (paper Sec. 2.1 stage 5, Sec. 6), different tiling: whole Q rows of 32 positives and
// whole rows of 32 negatives fit LDS together, the score tile is a single 32x32 MFMA block
// whose contraction over the dimension is split across the four waves (partials summed
// through LDS), and each wave owns up to four 32-wide column blocks of the two gradient
// products.
#include <type_traits>

#include "chunk_common.h"

namespace legend {

constexpr int kWT = kWideRowTile;       // positives per workgroup and negatives per tile
constexpr int kWSw = 36;                // row stride of the 32x32 score / W tiles
constexpr int kWideItems = 16;          // float4 per thread of one gathered tile (32 rows x 512 floats / 256 threads)

template <int SCORE, int LOSS>
__global__ void __launch_bounds__(kChunkThreads, 1)
k_chunk_wide(BatchGeom g, BucketParams bp, const int32_t* __restrict__ neg_ids, float* __restrict__ grad,
             double* __restrict__ loss_partial) {
    extern __shared__ __align__(16) float smem[];
    const int d = bp.dim;
    const int V4 = d >> 2;                      // float4 per row
    const int QS = chunk_row_stride(d);
    const int G_d = (d + 7) >> 3;
    const int NBW = (d + 31) >> 5;              // 32-wide column blocks
    const int tile_floats = kWT * QS + 32;
    float* Qs = smem;                           // [32][QS]
    float* Ns = Qs + tile_floats;               // [32][QS]  negative tile, later staging / G_Q
    float* Sp = Ns + tile_floats;               // [4][32][36] per-wave partial scores
    float* Ws = Sp + 4 * kWT * kWSw;            // [32][36]  W of the tile
    float* pos_s = Ws + kWT * kWSw;             // [32]
    float* lse_s = pos_s + kWT;                 // [32]
    float* rowloss_s = lse_s + kWT;             // [32]
    int32_t* ids_s = reinterpret_cast<int32_t*>(rowloss_s + kWT);   // [kIdsLds]

    const int tid = threadIdx.x;
    const int w = tid >> 6;
    const int lane = tid & 63;
    const int i32 = lane & 31;
    const int kk = lane >> 5;

    int wg = blockIdx.x;
    const int t = wg % g.T;  wg /= g.T;
    const int c = wg % g.nchunks;
    const int si = wg / g.nchunks;
    const int side = g.side_id[si];
    const int chunk_rows = min(g.C, g.P - c * g.C);
    const int row0 = t * g.rows_tile;
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
    const int64_t neg_base = side_base + (int64_t)g.roles * g.P + ((int64_t)c * g.T + t) * N;
    const bool atomic = bp.atomic_mode != 0;

    for (int k = tid; k < min(N, kIdsLds); k += kChunkThreads) ids_s[k] = my_negs[k];
    for (int idx = tid; idx < kWT * (QS - d); idx += kChunkThreads) {
        int r = idx / (QS - d), cc = d + idx % (QS - d);
        Qs[r * QS + cc] = 0.f;
        Ns[r * QS + cc] = 0.f;
    }

    // ---- prologue: 8 threads per positive ---------------------------------------------------
    const int prow = tid >> 3;
    const int ppart = tid & 7;
    {
        float partial = 0.f;
        if (prow < nrows) {
            const float* x = Ex + (int64_t)eb[prow * 3 + xcol] * d;
            const float* y = Ey + (int64_t)eb[prow * 3 + ycol] * d;
            const float* r = SCORE == LEGEND_SCORE_DOT ? x : bp.E_rel + (int64_t)eb[prow * 3 + 1] * d;
            if (SCORE == LEGEND_SCORE_COMPLEX) {
                const int h = d >> 1;
                for (int k = ppart; k < h; k += 8) {
                    float xr = x[k], xi = x[k + h], rr = r[k], ri = r[k + h];
                    float qr, qi;
                    if (side == 0) { qr = xr * rr - xi * ri; qi = xr * ri + xi * rr; }
                    else           { qr = rr * xr + ri * xi; qi = rr * xi - ri * xr; }
                    Qs[prow * QS + k] = qr;
                    Qs[prow * QS + k + h] = qi;
                    partial += qr * y[k] + qi * y[k + h];
                }
            } else {
                for (int k = ppart; k < d; k += 8) {
                    float q = SCORE == LEGEND_SCORE_DOT ? x[k] : x[k] * r[k];
                    Qs[prow * QS + k] = q;
                    partial += q * y[k];
                }
            }
        } else {
            for (int k = ppart; k < d; k += 8) Qs[prow * QS + k] = 0.f;
        }
        partial += wave_shfl_xor(partial, 1);
        partial += wave_shfl_xor(partial, 2);
        partial += wave_shfl_xor(partial, 4);
        if (ppart == 0) pos_s[prow] = partial;
    }
    __syncthreads();

    // ---- gather of a 32-row negative tile: item s of a thread is float4 number tid + 256 s ----
    const int F = kWT * V4;
    const int step_row = kChunkThreads / V4, step_col = kChunkThreads % V4;
    const bool ids_in_lds = N <= kIdsLds;
    float4 pf[kWideItems];
    auto for_items = [&](auto&& fn) {
        int row = tid / V4, c4 = tid % V4;
#pragma unroll
        for (int s = 0; s < kWideItems; ++s) {
            fn(s, tid + kChunkThreads * s < F, row, c4);
            row += step_row;
            c4 += step_col;
            if (c4 >= V4) { c4 -= V4; ++row; }
        }
    };
    auto gather_issue = [&](int n0) {
        for_items([&](int s, bool live, int row, int c4) {
            const int rr = live ? row : 0, cc = live ? c4 : 0;
            const int k = min(n0 + rr, N - 1);
            typedef __attribute__((address_space(3))) const int32_t* lds_ids_t;
            int32_t id;
            if (ids_in_lds) id = ((lds_ids_t)ids_s)[k];
            else id = my_negs[k];
            pf[s] = *reinterpret_cast<const float4*>(En + (int64_t)id * d + 4 * cc);
        });
    };
    auto gather_commit = [&](int n0) {
        for_items([&](int s, bool live, int row, int c4) {
            if (live) {
                float4 v = pf[s];
                if (n0 + row >= N) v = make_float4(0.f, 0.f, 0.f, 0.f);
                *reinterpret_cast<float4*>(Ns + row * QS + 4 * c4) = v;
            }
        });
    };
    auto acc_row = [&](int v) { return 8 * (v >> 2) + 4 * kk + (v & 3); };

    // ---- score tile: each wave contracts its share of the dimension, partials go to LDS -------
    auto score_partial = [&]() {
        f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        const float* qa = Qs + i32 * QS + 4 * kk;
        const float* nb = Ns + i32 * QS + 4 * kk;
        for (int gi = w; gi < G_d; gi += 4) {
            const float4 a = lds4(qa + 8 * gi), b = lds4(nb + 8 * gi);
            acc = mfma32(a.x, b.x, acc);
            acc = mfma32(a.y, b.y, acc);
            acc = mfma32(a.z, b.z, acc);
            acc = mfma32(a.w, b.w, acc);
        }
        float* sp = Sp + w * kWT * kWSw;
#pragma unroll
        for (int v = 0; v < 16; ++v) sp[acc_row(v) * kWSw + i32] = acc[v];
    };
    // the thread's four scores of row prow (columns 4*ppart .. +3): sum of the four partials
    auto score_of_thread = [&]() -> float4 {
        const float* p = Sp + prow * kWSw + 4 * ppart;
        float4 s0 = lds4(p), s1 = lds4(p + kWT * kWSw), s2 = lds4(p + 2 * kWT * kWSw), s3 = lds4(p + 3 * kWT * kWSw);
        return make_float4((s0.x + s1.x) + (s2.x + s3.x), (s0.y + s1.y) + (s2.y + s3.y),
                           (s0.z + s1.z) + (s2.z + s3.z), (s0.w + s1.w) + (s2.w + s3.w));
    };

    const int ntiles = (N + kWT - 1) / kWT;
    float lse = 0.f;
    float neg_loss = 0.f;

    gather_issue(0);
    if (LOSS == LEGEND_LOSS_SOFTMAX) {
        // ---- sweep 1: log-sum-exp per row; the 8 threads of a row keep identical (max, sum) ----
        float m_run = -INFINITY, l_run = 0.f;
        for (int tile = 0; tile < ntiles; ++tile) {
            const int n0 = tile * kWT;
            gather_commit(n0);
            __syncthreads();
            gather_issue(tile + 1 < ntiles ? n0 + kWT : 0);
            score_partial();
            __syncthreads();
            const float4 sv = score_of_thread();
            const float sa[4] = {sv.x, sv.y, sv.z, sv.w};
            const int ncol = min(4, N - n0 - 4 * ppart);
            float tmax = -INFINITY;
#pragma unroll
            for (int j = 0; j < 4; ++j) if (j < ncol) tmax = fmaxf(tmax, sa[j]);
            tmax = fmaxf(tmax, wave_shfl_xor(tmax, 1));
            tmax = fmaxf(tmax, wave_shfl_xor(tmax, 2));
            tmax = fmaxf(tmax, wave_shfl_xor(tmax, 4));
            const float m_new = fmaxf(m_run, tmax);
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) if (j < ncol) sum += fast_exp(sa[j] - m_new);
            sum += wave_shfl_xor(sum, 1);
            sum += wave_shfl_xor(sum, 2);
            sum += wave_shfl_xor(sum, 4);
            l_run = l_run * expf(m_run - m_new) + sum;
            m_run = m_new;
            // the partial tiles are rewritten only after the next commit's barrier
        }
        lse = m_run + logf(l_run);
        if (bp.softmax_with_pos) {            // the positive score joins the log-sum-exp
            const float f = pos_s[prow];
            const float hi = fmaxf(lse, f), lo = fminf(lse, f);
            lse = hi + log1pf(expf(lo - hi));
        }
        if (ppart == 0) lse_s[prow] = lse;
    }

    // ---- sweep 2 ------------------------------------------------------------------------------
    f32x16 accB[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) accB[j][v] = 0.f;
    const int nj = w < NBW ? (NBW - w + 3) / 4 : 0;     // column blocks of this wave: w, w+4, ...
    const int G_rows = (nrows + 7) >> 3;
    const float wneg = bp.neg_weight;
    f32x16 accC[4];

    auto products = [&](auto NJ, int n0) {
        constexpr int J = decltype(NJ)::value;
        const int G_n = (min(kWT, N - n0) + 7) >> 3;
        {   // G_Q += W * Neg
            const float* wa = Ws + i32 * kWSw + 4 * kk;
            const float* nb = Ns + (4 * kk) * QS + w * 32 + i32;
            for (int gi = 0; gi < G_n; ++gi) {
                const float4 a = lds4(wa + 8 * gi);
                const float* nbg = nb + 8 * gi * QS;
                float b[J][4];
#pragma unroll
                for (int j = 0; j < J; ++j)
#pragma unroll
                    for (int s = 0; s < 4; ++s) b[j][s] = nbg[s * QS + 128 * j];
#pragma unroll
                for (int j = 0; j < J; ++j) {
                    accB[j] = mfma32(a.x, b[j][0], accB[j]);
                    accB[j] = mfma32(a.y, b[j][1], accB[j]);
                    accB[j] = mfma32(a.z, b[j][2], accB[j]);
                    accB[j] = mfma32(a.w, b[j][3], accB[j]);
                }
            }
        }
        {   // G_neg = W^T * Q
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) accC[j][v] = 0.f;
            const float* wa = Ws + (4 * kk) * kWSw + i32;
            const float* qb = Qs + (4 * kk) * QS + w * 32 + i32;
            for (int gi = 0; gi < G_rows; ++gi) {
                const float* wag = wa + 8 * gi * kWSw;
                const float* qbg = qb + 8 * gi * QS;
                float a[4], b[J][4];
#pragma unroll
                for (int s = 0; s < 4; ++s) a[s] = wag[s * kWSw];
#pragma unroll
                for (int j = 0; j < J; ++j)
#pragma unroll
                    for (int s = 0; s < 4; ++s) b[j][s] = qbg[s * QS + 128 * j];
#pragma unroll
                for (int j = 0; j < J; ++j)
#pragma unroll
                    for (int s = 0; s < 4; ++s) accC[j] = mfma32(a[s], b[j][s], accC[j]);
            }
        }
    };
    auto stage_blocks = [&](auto NJ, float* dst, const f32x16* acc) {
        constexpr int J = decltype(NJ)::value;
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int col = (w + 4 * j) * 32 + i32;
            if (col < d) {
#pragma unroll
                for (int v = 0; v < 16; ++v) dst[acc_row(v) * QS + col] = acc[j][v];
            }
        }
    };
    using J1 = std::integral_constant<int, 1>;
    using J2 = std::integral_constant<int, 2>;
    using J3 = std::integral_constant<int, 3>;
    using J4 = std::integral_constant<int, 4>;

    for (int tile = 0; tile < ntiles; ++tile) {
        const int n0 = tile * kWT;
        gather_commit(n0);
        __syncthreads();
        if (tile + 1 < ntiles) gather_issue(n0 + kWT);
        score_partial();
        __syncthreads();
        {
            const float4 sv = score_of_thread();
            const float sa[4] = {sv.x, sv.y, sv.z, sv.w};
            const int ncol = prow < nrows ? min(4, N - n0 - 4 * ppart) : 0;
            float wv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                wv[j] = 0.f;
                if (j < ncol) {
                    if (LOSS == LEGEND_LOSS_SOFTMAX) {
                        wv[j] = fast_exp(sa[j] - lse);
                    } else {
                        wv[j] = wneg * sigmoidf(sa[j]);
                        neg_loss += wneg * softplusf(sa[j]);
                    }
                }
            }
            *reinterpret_cast<float4*>(Ws + prow * kWSw + 4 * ppart) = make_float4(wv[0], wv[1], wv[2], wv[3]);
        }
        __syncthreads();
        switch (nj) {
            case 1: products(J1{}, n0); break;
            case 2: products(J2{}, n0); break;
            case 3: products(J3{}, n0); break;
            case 4: products(J4{}, n0); break;
            default: break;
        }
        __syncthreads();                      // the negative tile is not read any more
        switch (nj) {
            case 1: stage_blocks(J1{}, Ns, accC); break;
            case 2: stage_blocks(J2{}, Ns, accC); break;
            case 3: stage_blocks(J3{}, Ns, accC); break;
            case 4: stage_blocks(J4{}, Ns, accC); break;
            default: break;
        }
        __syncthreads();
        {
            float* Gn = side == 0 ? bp.G_dst : bp.G_src;
            for_items([&](int s, bool live, int row, int c4) {
                const int neg = n0 + row;
                if (live && neg < N) {
                    const float4 v = lds4(Ns + row * QS + 4 * c4);
                    if (atomic) {
                        const int32_t id = neg < kIdsLds ? ids_s[neg] : my_negs[neg];
                        float* dst = Gn + (int64_t)id * d + 4 * c4;
                        unsafeAtomicAdd(dst, v.x);
                        unsafeAtomicAdd(dst + 1, v.y);
                        unsafeAtomicAdd(dst + 2, v.z);
                        unsafeAtomicAdd(dst + 3, v.w);
                    } else {
                        *reinterpret_cast<float4*>(grad + (neg_base + neg) * d + 4 * c4) = v;
                    }
                }
            });
        }
        __syncthreads();
    }

    // ---- epilogue -----------------------------------------------------------------------------
    float* Gs = Ns;
    switch (nj) {
        case 1: stage_blocks(J1{}, Gs, accB); break;
        case 2: stage_blocks(J2{}, Gs, accB); break;
        case 3: stage_blocks(J3{}, Gs, accB); break;
        case 4: stage_blocks(J4{}, Gs, accB); break;
        default: break;
    }
    if (LOSS == LEGEND_LOSS_LOGISTIC) {
        for (int off = kWave / 2; off > 0; off >>= 1) neg_loss += __shfl_down(neg_loss, off, kWave);
        if (lane == 0) lse_s[w] = neg_loss;
    }
    __syncthreads();
    auto emit = [&](float* p, float v) {
        if (atomic) unsafeAtomicAdd(p, v);
        else *p = v;
    };
    {
        float row_loss = 0.f;
        if (prow < nrows) {
            const float f = pos_s[prow];
            float a;
            if (LOSS == LEGEND_LOSS_SOFTMAX) {
                row_loss = lse - f;
                a = bp.softmax_with_pos ? expf(-row_loss) - 1.f : -1.f;
            }
            else { a = -sigmoidf(-f); row_loss = softplusf(-f); }
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
            const float* q = Qs + prow * QS;
            if (SCORE == LEGEND_SCORE_COMPLEX) {
                const int h = d >> 1;
                for (int k = ppart; k < h; k += 8) {
                    float gre = gq[k] + a * y[k], gim = gq[k + h] + a * y[k + h];
                    float xr = x[k], xi = x[k + h], rr = r[k], ri = r[k + h];
                    emit(gy + k, a * q[k]);
                    emit(gy + k + h, a * q[k + h]);
                    if (side == 0) {
                        emit(gx + k, rr * gre + ri * gim);      emit(gx + k + h, rr * gim - ri * gre);
                        emit(gr + k, xr * gre + xi * gim);      emit(gr + k + h, xr * gim - xi * gre);
                    } else {
                        emit(gx + k, rr * gre - ri * gim);      emit(gx + k + h, rr * gim + ri * gre);
                        emit(gr + k, gre * xr + gim * xi);      emit(gr + k + h, gre * xi - gim * xr);
                    }
                }
            } else {
                for (int k = ppart; k < d; k += 8) {
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
        for (int r = 0; r < kWT; ++r) s += (double)rowloss_s[r];
        if (LOSS == LEGEND_LOSS_LOGISTIC)
            for (int ww = 0; ww < kChunkThreads / kWave; ++ww) s += (double)lse_s[ww];
        loss_partial[blockIdx.x] = s;
    }
}

static size_t wide_lds_bytes(int d) {
    const int QS = chunk_row_stride(d);
    size_t floats = 2 * ((size_t)kWT * QS + 32) + 5 * (size_t)kWT * kWSw + 3 * kWT + kIdsLds;
    return floats * sizeof(float);
}

hipError_t launch_chunks_wide(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    if (bp.dim <= kNarrowMaxDim || bp.dim > kWideMaxDim || (bp.dim & 3)) return hipErrorInvalidValue;
    dim3 grid((unsigned)(g.sides * g.nchunks * g.T)), block(kChunkThreads);
    const size_t lds = wide_lds_bytes(bp.dim);
#define LEGEND_WIDE_CASE(SC, LO)                                                                               \
    if (bp.score == SC && bp.loss == LO) {                                                                     \
        static size_t lds_allowed = 0;                                                                         \
        if (lds > lds_allowed) {                                                                               \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_chunk_wide<SC, LO>),           \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
            if (e != hipSuccess) return e;                                                                     \
            lds_allowed = lds;                                                                                 \
        }                                                                                                      \
        hipLaunchKernelGGL((k_chunk_wide<SC, LO>), grid, block, lds, st, g, bp, ws.neg_ids, ws.grad,           \
                           ws.loss_partial);                                                                   \
        return hipGetLastError();                                                                              \
    }
    LEGEND_WIDE_CASE(LEGEND_SCORE_DOT, LEGEND_LOSS_SOFTMAX)
    LEGEND_WIDE_CASE(LEGEND_SCORE_DOT, LEGEND_LOSS_LOGISTIC)
    LEGEND_WIDE_CASE(LEGEND_SCORE_DISTMULT, LEGEND_LOSS_SOFTMAX)
    LEGEND_WIDE_CASE(LEGEND_SCORE_DISTMULT, LEGEND_LOSS_LOGISTIC)
    LEGEND_WIDE_CASE(LEGEND_SCORE_COMPLEX, LEGEND_LOSS_SOFTMAX)
    LEGEND_WIDE_CASE(LEGEND_SCORE_COMPLEX, LEGEND_LOSS_LOGISTIC)
#undef LEGEND_WIDE_CASE
    return hipErrorInvalidValue;
}

}  // namespace legend
