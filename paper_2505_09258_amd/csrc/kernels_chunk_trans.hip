// Chunk computation for the translational score (Sec. 8 names such models as easy to add; Sec. 6's
// frame (theta_s (x) theta_r) (+) theta_d with (x) an addition and (+) a negative L1 distance):
//   q = theta_x + theta_r (destination side) or theta_x - theta_r (source side), an fp32 number;
//   score of q against a row y: -|q - y|_1;  d score/dq = -sign(q - y), d score/dy = +sign(q - y).
// The negative block is no matrix product, so nothing here uses the matrix pipe: the kernel is
// bound by vector ALU throughput.  Two sweeps over the chunk's negatives in tiles of 64, as in the
// general kernel for the product scores: the first takes the row-wise log-sum-exp (skipped for the
// logistic and margin losses), the second recomputes the scores, forms W = dL/dS and accumulates
//   G_q[e] -= W[e][k] sign(q_e - n_k),   G_neg[k] += W[e][k] sign(q_e - n_k)
// from one evaluation of every sign.
#include <hip/hip_runtime.h>

#include "chunk_common.h"

namespace legend {

namespace {

constexpr int kTRows = 64;          // positives per workgroup
constexpr int kTNeg = 64;           // negatives per tile
constexpr int kTWS = 68;            // row stride of the transposed W tile
constexpr int kTThreads = 256;

// w * sign(diff) for w >= 0, sign(0) = 0
__device__ inline float sign_times(float diff, float w) {
    const float t = __builtin_copysignf(w, diff);
    return diff == 0.f ? 0.f : t;
}
// Sum over the eight lanes 8j..8j+7 of a wave, valid in lane 8j (and 8j+7): data-parallel
// primitives within a row of 16 lanes (two quad permutations, then the mirror of each half row).
__device__ inline float sum8(float v) {
    int x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, true));   // row_half_mirror
    return v;
}
__device__ inline float l1_of(float4 a, float4 b) {
    return (fabsf(a.x - b.x) + fabsf(a.y - b.y)) + (fabsf(a.z - b.z) + fabsf(a.w - b.w));
}

template <int LOSS>
__global__ void __launch_bounds__(kTThreads, 2)
k_chunk_trans(BatchGeom g, BucketParams bp, const int32_t* __restrict__ neg_ids, float* __restrict__ grad,
              double* __restrict__ loss_partial) {
    extern __shared__ __align__(16) float smem[];
    const int d = bp.dim;
    const int QS = chunk_row_stride(d);
    const int d4 = (d + 3) >> 2;
    float* Qs = smem;                          // [64][QS] q rows
    float* Ns = Qs + kTRows * QS;              // [64][QS] current negative tile (later: G_q)
    float* Wt = Ns + kTNeg * QS;               // [64 negatives][68] W of the current tile, transposed
    float* pos_s = Wt + kTNeg * kTWS;          // [64]
    float* lse_s = pos_s + kTRows;             // [64]
    float* rowloss_s = lse_s + kTRows;         // [64]

    const int tid = threadIdx.x;
    int wg = blockIdx.x;
    const int t = wg % g.T;  wg /= g.T;
    const int c = wg % g.nchunks;
    const int si = wg / g.nchunks;
    const int side = g.side_id[si];            // 0: destination corrupted, 1: source corrupted
    const int chunk_rows = min(g.C, g.P - c * g.C);
    const int row0 = t * g.rows_tile;
    const int nrows = max(0, min(g.rows_tile, chunk_rows - row0));
    const int64_t e0 = (int64_t)c * g.C + row0;
    const int32_t* eb = bp.edges + (bp.batch_lo + e0) * 3;
    const float* Ex = side == 0 ? bp.E_src : bp.E_dst;          // rows combined with the relation
    const float* Ey = side == 0 ? bp.E_dst : bp.E_src;          // rows that meet q; negatives replace them
    const int xcol = side == 0 ? 0 : 2;
    const int ycol = 2 - xcol;
    const int N = g.N;
    const int32_t* my_negs = neg_ids + ((int64_t)si * g.nchunks + c) * N;
    const int64_t side_base = (int64_t)si * g.per_side;
    const int64_t neg_base = side_base + (int64_t)g.roles * g.P + ((int64_t)c * g.T + t) * N;
    const bool vec4 = (d & 3) == 0;
    const float rsign = side == 0 ? 1.f : -1.f;                 // q = x + r or x - r

    // ---- prologue: q rows (zero beyond d and beyond nrows) and positive scores; 4 threads per row
    const int prow = tid >> 2;
    const int ppart = tid & 3;
    {
        float partial = 0.f;
        if (prow < nrows) {
            const float* x = Ex + (int64_t)eb[prow * 3 + xcol] * d;
            const float* y = Ey + (int64_t)eb[prow * 3 + ycol] * d;
            const float* r = bp.E_rel + (int64_t)eb[prow * 3 + 1] * d;
            for (int k = ppart; k < QS; k += 4) {
                float q = 0.f;
                if (k < d) {
                    q = x[k] + rsign * r[k];
                    partial += fabsf(q - y[k]);
                }
                Qs[prow * QS + k] = q;
            }
        } else {
            for (int k = ppart; k < QS; k += 4) Qs[prow * QS + k] = 0.f;
        }
        partial += wave_shfl_xor(partial, 1);
        partial += wave_shfl_xor(partial, 2);
        if (ppart == 0) pos_s[prow] = -partial;
    }

    // negative tile n0..n0+63 into Ns; rows past N and columns past d are zero
    auto gather_tile = [&](int n0) {
        for (int idx = tid; idx < kTNeg * (QS / 4); idx += kTThreads) {
            const int rt = idx / (QS / 4), c4 = idx % (QS / 4);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (n0 + rt < N && c4 < d4) {
                const float* src = Ey + (int64_t)my_negs[n0 + rt] * d + 4 * c4;
                if (vec4) {
                    v = *reinterpret_cast<const float4*>(src);
                } else {
                    v.x = src[0];
                    if (4 * c4 + 1 < d) v.y = src[1];
                    if (4 * c4 + 2 < d) v.z = src[2];
                    if (4 * c4 + 3 < d) v.w = src[3];
                }
            }
            *reinterpret_cast<float4*>(Ns + rt * QS + 4 * c4) = v;
        }
    };
    // scores of rows 4ty..4ty+3 against negatives tx, tx+16, tx+32, tx+48 of the tile
    const int ty = tid >> 4, tx = tid & 15;
    auto score_block = [&](float (&S)[4][4]) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) S[a][b] = 0.f;
        for (int j4 = 0; j4 < d4; ++j4) {
            float4 q4[4], n4[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) q4[a] = lds4(Qs + (4 * ty + a) * QS + 4 * j4);
#pragma unroll
            for (int b = 0; b < 4; ++b) n4[b] = lds4(Ns + (tx + 16 * b) * QS + 4 * j4);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) S[a][b] += l1_of(q4[a], n4[b]);
        }
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) S[a][b] = -S[a][b];
    };
    const int ntiles = (N + kTNeg - 1) / kTNeg;

    // ---- sweep 1: row-wise log-sum-exp over the negatives (softmax only) ----------------------
    if (LOSS == LEGEND_LOSS_SOFTMAX) {
        float m[4], l[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) { m[a] = -INFINITY; l[a] = 0.f; }
        for (int tile = 0; tile < ntiles; ++tile) {
            __syncthreads();                  // the previous tile (and, first, Qs) is no longer written / read
            gather_tile(tile * kTNeg);
            __syncthreads();
            float S[4][4];
            score_block(S);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (tile * kTNeg + tx + 16 * b < N) {
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const float mn = fmaxf(m[a], S[a][b]);
                        l[a] = l[a] * expf(m[a] - mn) + expf(S[a][b] - mn);
                        m[a] = mn;
                    }
                }
            }
        }
        // the 16 lanes tx = 0..15 of a row group hold disjoint columns of the same four rows
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int mask = 1; mask < 16; mask <<= 1) {
                const float mo = wave_shfl_xor(m[a], mask), lo = wave_shfl_xor(l[a], mask);
                const float mn = fmaxf(m[a], mo);
                if (mn > -INFINITY) l[a] = l[a] * expf(m[a] - mn) + lo * expf(mo - mn);
                m[a] = mn;
            }
            if (tx == 0) {
                float mm = m[a], ll = l[a];
                if (bp.softmax_with_pos) {     // Eq. 1 variant: the positive score is one more term
                    const float f = pos_s[4 * ty + a];
                    // lse over the negatives - f: the loss term is its softplus and dL/df minus its sigmoid
                    rowloss_s[4 * ty + a] = mm + logf(ll) - f;
                    const float mn = fmaxf(mm, f);
                    ll = (mm > -INFINITY ? ll * expf(mm - mn) : 0.f) + expf(f - mn);
                    mm = mn;
                }
                lse_s[4 * ty + a] = mm + logf(ll);
            }
        }
    }

    // ---- sweep 2: W, G_q and G_neg --------------------------------------------------------------
    // gradient pass: 8 lanes (rb = 0..7) share the four columns 4jg..4jg+3; lane rb owns rows
    // rb, rb + 8, ..., so that the row groups past the chunk's last row drop out for all lanes at once
    const int rb = tid & 7, jg = tid >> 3;
    const bool gactive = jg < d4;
    const int imax = (nrows + 7) >> 3;
    float4 accq[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) accq[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    float neg_loss = 0.f;
    float hinge[4] = {0.f, 0.f, 0.f, 0.f}, viol[4] = {0.f, 0.f, 0.f, 0.f};    // margin loss: rows 4ty..4ty+3 over this lane's columns
    const bool atomic = bp.atomic_mode != 0;
    float* Gn = side == 0 ? bp.G_dst : bp.G_src;
    for (int tile = 0; tile < ntiles; ++tile) {
        const int n0 = tile * kTNeg;
        __syncthreads();                      // Ns and Wt of the previous tile are no longer read; lse_s is complete
        gather_tile(n0);
        __syncthreads();
        {
            float S[4][4];
            score_block(S);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const bool kvalid = n0 + tx + 16 * b < N;
                float w4[4];
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const bool valid = kvalid && 4 * ty + a < nrows;
                    float w = 0.f;
                    if (valid) {
                        if (LOSS == LEGEND_LOSS_SOFTMAX) {
                            w = expf(S[a][b] - lse_s[4 * ty + a]);
                        } else if (LOSS == LEGEND_LOSS_MARGIN) {
                            // the pair pays margin - f + S where that is positive; W is the indicator
                            const float sh = (bp.margin - pos_s[4 * ty + a]) + S[a][b];
                            w = sh > 0.f ? 1.f : 0.f;
                            hinge[a] += fmaxf(sh, 0.f);
                            viol[a] += w;
                        } else {
                            w = bp.neg_weight * sigmoidf(S[a][b]);
                            neg_loss += bp.neg_weight * softplusf(S[a][b]);
                        }
                    }
                    w4[a] = w;
                }
                // row r sits at position (r % 8) * 8 + r / 8: the eight rows of a lane of the gradient pass are adjacent
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const int r = 4 * ty + a;
                    Wt[(tx + 16 * b) * kTWS + (r & 7) * 8 + (r >> 3)] = w4[a];
                }
            }
        }
        __syncthreads();
        if (gactive) {
            float4 q[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) q[i] = lds4(Qs + (rb + 8 * i) * QS + 4 * jg);
            for (int k = 0; k < kTNeg; ++k) {
                const float4 n4 = lds4(Ns + k * QS + 4 * jg);
                const float4 wa = lds4(Wt + k * kTWS + 8 * rb), wb = lds4(Wt + k * kTWS + 8 * rb + 4);
                const float w8[8] = {wa.x, wa.y, wa.z, wa.w, wb.x, wb.y, wb.z, wb.w};
                float4 pn = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (i < imax) {
                        float tv;
                        tv = sign_times(q[i].x - n4.x, w8[i]); accq[i].x -= tv; pn.x += tv;
                        tv = sign_times(q[i].y - n4.y, w8[i]); accq[i].y -= tv; pn.y += tv;
                        tv = sign_times(q[i].z - n4.z, w8[i]); accq[i].z -= tv; pn.z += tv;
                        tv = sign_times(q[i].w - n4.w, w8[i]); accq[i].w -= tv; pn.w += tv;
                    }
                }
                // the rows of the eight lanes of the group, in a fixed order
                pn.x = sum8(pn.x);
                pn.y = sum8(pn.y);
                pn.z = sum8(pn.z);
                pn.w = sum8(pn.w);
                if (rb == 0 && n0 + k < N) {
                    const int col = 4 * jg;
                    if (atomic) {
                        float* dst = Gn + (int64_t)my_negs[n0 + k] * d + col;
                        unsafeAtomicAdd(dst, pn.x);
                        if (col + 1 < d) unsafeAtomicAdd(dst + 1, pn.y);
                        if (col + 2 < d) unsafeAtomicAdd(dst + 2, pn.z);
                        if (col + 3 < d) unsafeAtomicAdd(dst + 3, pn.w);
                    } else {
                        float* dst = grad + (neg_base + n0 + k) * d + col;
                        if (vec4) {
                            *reinterpret_cast<float4*>(dst) = pn;
                        } else {
                            dst[0] = pn.x;
                            if (col + 1 < d) dst[1] = pn.y;
                            if (col + 2 < d) dst[2] = pn.z;
                            if (col + 3 < d) dst[3] = pn.w;
                        }
                    }
                }
            }
        }
    }

    // ---- epilogue: G_q to LDS, positive terms, chain rule, gradient rows of the positives -------
    __syncthreads();                          // the last tile is no longer read
    float* Gs = Ns;
    if (gactive) {
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<float4*>(Gs + (rb + 8 * i) * QS + 4 * jg) = accq[i];
    }
    if (LOSS == LEGEND_LOSS_LOGISTIC) {
        for (int off = kWave / 2; off > 0; off >>= 1) neg_loss += __shfl_down(neg_loss, off, kWave);
        if ((tid & 63) == 0) lse_s[tid >> 6] = neg_loss;
    }
    if (LOSS == LEGEND_LOSS_MARGIN) {
        // the 16 lanes tx = 0..15 of a row group hold disjoint columns of the same four rows
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int mask = 1; mask < 16; mask <<= 1) {
                hinge[a] += wave_shfl_xor(hinge[a], mask);
                viol[a] += wave_shfl_xor(viol[a], mask);
            }
            if (tx == 0) {
                lse_s[4 * ty + a] = hinge[a];         // the row's loss term
                rowloss_s[4 * ty + a] = viol[a];      // how many of its negatives pay: -dL/df
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
            } else if (LOSS == LEGEND_LOSS_MARGIN) {
                a = -rowloss_s[prow];                         // read by the row's four lanes before one of them reuses the slot
                row_loss = lse_s[prow];
            } else {
                a = -sigmoidf(-f);
                row_loss = softplusf(-f);
            }
            const float* y = Ey + (int64_t)eb[prow * 3 + ycol] * d;
            const int64_t e = e0 + prow;
            float* gx = grad + (side_base + (side == 0 ? 0 : g.P) + e) * d;        // source rows first
            float* gy = grad + (side_base + (side == 0 ? g.P : 0) + e) * d;
            float* gr = grad + (side_base + 2 * (int64_t)g.P + e) * d;
            if (atomic) {
                gx = (side == 0 ? bp.G_src : bp.G_dst) + (int64_t)eb[prow * 3 + xcol] * d;
                gy = (side == 0 ? bp.G_dst : bp.G_src) + (int64_t)eb[prow * 3 + ycol] * d;
                gr = bp.G_rel + (int64_t)eb[prow * 3 + 1] * d;
            }
            for (int k = ppart; k < d; k += 4) {
                const float sp = a * sign_times(Qs[prow * QS + k] - y[k], 1.f);  // a * sign(q - y)
                const float gq = Gs[prow * QS + k] - sp;
                emit(gy + k, sp);
                emit(gx + k, gq);
                emit(gr + k, rsign * gq);
            }
        }
        if (ppart == 0) rowloss_s[prow] = row_loss;
    }
    __syncthreads();
    if (tid == 0) {
        double s = 0.0;
        for (int r = 0; r < kTRows; ++r) s += (double)rowloss_s[r];
        if (LOSS == LEGEND_LOSS_LOGISTIC)
            for (int ww = 0; ww < kTThreads / kWave; ++ww) s += (double)lse_s[ww];
        loss_partial[blockIdx.x] = s;
    }
}

template <int LOSS>
hipError_t launch_trans(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    const int QS = chunk_row_stride(bp.dim);
    const size_t lds = sizeof(float) * ((size_t)(kTRows + kTNeg) * QS + (size_t)kTNeg * kTWS + 3 * kTRows);
    static size_t lds_allowed[64] = {};       // dynamic LDS above 64 KB has to be requested per kernel and per device
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
    if (dev < 0 || lds > lds_allowed[dev]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_chunk_trans<LOSS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        if (dev >= 0) lds_allowed[dev] = lds;
    }
    hipLaunchKernelGGL(k_chunk_trans<LOSS>, dim3((unsigned)(g.sides * g.nchunks * g.T)), dim3(kTThreads), lds, st, g, bp,
                       ws.neg_ids, ws.grad, ws.loss_partial);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_chunks_trans(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    if (bp.dim > kNarrowMaxDim || g.rows_tile > kTRows) return hipErrorInvalidValue;
    if (bp.loss == LEGEND_LOSS_LOGISTIC) return launch_trans<LEGEND_LOSS_LOGISTIC>(st, g, bp, ws);
    if (bp.loss == LEGEND_LOSS_MARGIN) return launch_trans<LEGEND_LOSS_MARGIN>(st, g, bp, ws);
    return launch_trans<LEGEND_LOSS_SOFTMAX>(st, g, bp, ws);
}

}  // namespace legend
