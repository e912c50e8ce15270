// Batch computation for wide embeddings (128 < dim <= 512; paper Sec. 2.1
// stage 5, Sec. 6) as a short chain of tiled fp32-MFMA contractions.  A (row tile of <= 112
// positives) x (all N negatives) score block does not fit on chip next to d-wide operand tiles,
// so the scores go through a device buffer that stays in the L2 / Infinity cache (the paper keeps
// its "Intermediate Result 3" in global memory for the same reason):
//   k_gemm_compose   Q = theta_s (x) theta_r (or conj(theta_r) (x) theta_d), positive scores f
//   k_gemm_scores    S = Q Neg^T, 112 x 64 tiles, the dimension streamed in slices of 80 columns
//   k_gemm_rowstats  per row: log-sum-exp, loss term, dL/df; S is replaced by the weights W = dL/dS
//   k_gemm_gq        G_Q = W Neg
//   k_gemm_gneg      G_neg = W^T Q, written to the gradient rows of the negatives
//   k_gemm_chain     chain rule: gradient rows of theta_s, theta_r, theta_d of the positives
// All contractions use 16x16x4 MFMA with the contraction index in groups of 16 (lane group g
// supplies k = 16G + 4g + s to four consecutive MFMAs), so a k-contiguous operand is one 128-bit
// LDS read per four MFMAs; operands whose contraction index is the slow one are read 32 bits at
// a time.
#include "chunk_common.h"

namespace legend {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x4 mfma16g(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

constexpr int kGRows = 112;              // rows of a tile of positives: seven 16-row blocks
constexpr int kGRowBlocks = kGRows / 16;
constexpr int kGNeg = 64;                // negatives per tile
constexpr int kGSlice = 80;              // columns of the dimension per slice: five 16-column blocks
constexpr int kGSS = kGSlice + 4;        // LDS row stride of a slice
constexpr int kGWS = kGNeg + 4;          // LDS row stride of a W tile

static_assert(kGRows == kWideRowTile, "tile geometry");

// Workgroup ids are dealt round-robin to the eight XCDs, each with its own L2.  The tiled
// kernels launch a one-dimensional grid of 8 * ceil(total / 8) workgroups and turn the hardware
// id into a virtual id such that consecutive virtual ids (the tiles that share a row tile's
// operands) run on the same XCD.  Returns false for the padding workgroups.
constexpr int kXcds = 8;
__host__ __device__ inline int64_t xcd_grid(int64_t total) { return (total + kXcds - 1) / kXcds * kXcds; }
__device__ inline bool xcd_tile(int64_t total, int nx, int* bx, int64_t* by) {
    const int64_t lin = blockIdx.x;
    const int64_t per = (total + kXcds - 1) / kXcds;
    const int64_t v = (lin % kXcds) * per + lin / kXcds;
    if (v >= total) return false;
    *bx = (int)(v % nx);
    *by = v / nx;
    return true;
}

struct TileCoord {
    int si, side, c, t_row, nrows;
    int64_t e0;          // first edge of the tile inside the batch
    int64_t wgrow;       // (si * nchunks + c) * T + t_row
};

__device__ inline TileCoord tile_coord(const BatchGeom& g, int64_t wgrow) {
    TileCoord tc;
    tc.wgrow = wgrow;
    int64_t q = wgrow;
    tc.t_row = (int)(q % g.T);  q /= g.T;
    tc.c = (int)(q % g.nchunks);
    tc.si = (int)(q / g.nchunks);
    tc.side = g.side_id[tc.si];
    const int chunk_rows = min(g.C, g.P - tc.c * g.C);
    const int row0 = tc.t_row * g.rows_tile;
    tc.nrows = max(0, min(g.rows_tile, chunk_rows - row0));
    tc.e0 = (int64_t)tc.c * g.C + row0;
    return tc;
}

// ---- Q and positive scores --------------------------------------------------------------------
// one workgroup of 128 threads per (side, edge)
template <int SCORE>
__global__ void __launch_bounds__(128)
k_gemm_compose(BatchGeom g, BucketParams bp, float* __restrict__ Q, float* __restrict__ fpos) {
    const int64_t idx = blockIdx.x;
    const int si = (int)(idx / g.P);
    const int64_t e = idx % g.P;
    const int side = g.side_id[si];
    const int d = bp.dim;
    const int32_t* eb = bp.edges + (bp.batch_lo + e) * 3;
    const float* x = (side == 0 ? bp.E_src : bp.E_dst) + (int64_t)eb[side == 0 ? 0 : 2] * d;
    const float* y = (side == 0 ? bp.E_dst : bp.E_src) + (int64_t)eb[side == 0 ? 2 : 0] * d;
    const float* r = SCORE == LEGEND_SCORE_DOT ? x : bp.E_rel + (int64_t)eb[1] * d;
    float* q = Q + idx * d;
    float partial = 0.f;
    if (SCORE == LEGEND_SCORE_COMPLEX) {
        const int h = d >> 1;
        for (int k = threadIdx.x; k < h; k += 128) {
            const float xr = x[k], xi = x[k + h], rr = r[k], ri = r[k + h];
            float qr, qi;
            if (side == 0) { qr = xr * rr - xi * ri; qi = xr * ri + xi * rr; }
            else           { qr = rr * xr + ri * xi; qi = rr * xi - ri * xr; }
            q[k] = qr;
            q[k + h] = qi;
            partial += qr * y[k] + qi * y[k + h];
        }
    } else {
        for (int k = threadIdx.x; k < d; k += 128) {
            const float v = SCORE == LEGEND_SCORE_DOT ? x[k] : x[k] * r[k];
            q[k] = v;
            partial += v * y[k];
        }
    }
    __shared__ float red[128];
    red[threadIdx.x] = partial;
    __syncthreads();
    for (int off = 64; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) fpos[idx] = red[0];
}

// A thread's share of a [rows][64] tile of W (from the buffer the row statistics left) and of a
// [64][80] tile of negatives, fetched into registers one tile ahead of their use.
template <int THREADS>
struct WTileRegs {
    static constexpr int V4 = kGNeg / 4;
    static constexpr int ITEMS = (kGRows * V4 + THREADS - 1) / THREADS;
    float4 v[ITEMS];
    // Wtile: start of the row tile's block; the 64-negative tile n0 / 64 is the contiguous piece [rows_tile][64]
    __device__ void fetch(const float* Wtile, int rows_tile, int nrows, int n0, int tid) {
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            const int idx = tid + THREADS * k;
            const int row = idx / V4, c4 = idx - row * V4;
            v[k] = row < nrows ? *reinterpret_cast<const float4*>(Wtile + ((int64_t)(n0 / kGNeg) * rows_tile + row) * kGNeg + 4 * c4)
                               : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    __device__ void store(float* Wt, int tid) const {
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            const int idx = tid + THREADS * k;
            const int row = idx / V4, c4 = idx - row * V4;
            if (row < kGRows) *reinterpret_cast<float4*>(Wt + row * kGWS + 4 * c4) = v[k];
        }
    }
};

template <int THREADS, int ROWS, int WIDTH = kGSlice>
struct SliceRegs {                            // [ROWS][WIDTH columns] of row-major fp32 rows, LDS row stride WIDTH + 4
    static constexpr int V4 = WIDTH / 4;
    static constexpr int ITEMS = (ROWS * V4 + THREADS - 1) / THREADS;
    float4 v[ITEMS];
    // row_ptr(row) gives the start of the row or nullptr for a row that does not exist
    template <class F>
    __device__ void fetch(F&& row_ptr, int c0, int d, int tid) {
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            const int idx = tid + THREADS * k;
            const int row = idx / V4, c4 = idx - row * V4;
            const float* p = row < ROWS ? row_ptr(row) : nullptr;
            const int c = c0 + 4 * c4;
            float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
            if (p && c < d) {
                if ((d & 3) == 0) {           // rows are 16-byte aligned only then
                    o = *reinterpret_cast<const float4*>(p + c);
                } else if ((d & 1) == 0) {    // 8-byte aligned rows: two 64-bit loads
                    const float2 a = *reinterpret_cast<const float2*>(p + c);
                    o.x = a.x; o.y = a.y;
                    if (c + 2 < d) {
                        const float2 b = *reinterpret_cast<const float2*>(p + c + 2);
                        o.z = b.x; o.w = b.y;
                    }
                } else {
                    o.x = p[c];
                    if (c + 1 < d) o.y = p[c + 1];
                    if (c + 2 < d) o.z = p[c + 2];
                    if (c + 3 < d) o.w = p[c + 3];
                }
            }
            v[k] = o;
        }
    }
    __device__ void store(float* T, int tid) const {
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            const int idx = tid + THREADS * k;
            const int row = idx / V4, c4 = idx - row * V4;
            if (row < ROWS) *reinterpret_cast<float4*>(T + row * (WIDTH + 4) + 4 * c4) = v[k];
        }
    }
};

// ---- S = Q Neg^T ---------------------------------------------------------------------------------
// grid: (negative tiles, row tiles).  Four waves; wave w owns negatives 16w..16w+15 of the tile
// and all row blocks.  S is stored as [row tile][64-negative tile][row][64], so that the tiles the
// later kernels load are contiguous.
template <int RB>                             // row blocks of 16 that the tile geometry needs
__global__ void __launch_bounds__(256, 2)
k_gemm_scores(BatchGeom g, BucketParams bp, const int32_t* __restrict__ neg_ids, const float* __restrict__ Q,
              float* __restrict__ S, int Npad, int nx, int64_t ny) {
    __shared__ __align__(16) float Qs[kGRows * kGSS];
    __shared__ __align__(16) float Ns[kGNeg * kGSS];
    __shared__ int32_t ids_s[kGNeg];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l15 = lane & 15, gq = lane >> 4;
    int bx;
    int64_t by;
    if (!xcd_tile((int64_t)nx * ny, nx, &bx, &by)) return;       // uniform
    const TileCoord tc = tile_coord(g, by);
    const int n0 = bx * kGNeg;
    const int N = g.N, d = bp.dim;
    const float* En = tc.side == 0 ? bp.E_dst : bp.E_src;
    const float* Qrows = Q + ((int64_t)tc.si * g.P + tc.e0) * d;
    const int32_t* my_negs = neg_ids + ((int64_t)tc.si * g.nchunks + tc.c) * N;
    if (tid < kGNeg) ids_s[tid] = my_negs[min(n0 + tid, N - 1)];
    __syncthreads();

    f32x4 acc[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int nrows = tc.nrows;
    auto q_row = [=](int row) -> const float* { return row < nrows ? Qrows + (int64_t)row * d : nullptr; };
    const int32_t* ids = ids_s;
    auto n_row = [=](int row) -> const float* { return n0 + row < N ? En + (int64_t)ids[row] * d : nullptr; };
    SliceRegs<256, kGRows> qr;
    SliceRegs<256, kGNeg> nr;
    qr.fetch(q_row, 0, d, tid);
    nr.fetch(n_row, 0, d, tid);
    for (int c0 = 0; c0 < d; c0 += kGSlice) {
        // slice of Q and of the negatives into LDS (zero beyond the rows / negatives / columns that
        // exist), the next slice in flight
        qr.store(Qs, tid);
        nr.store(Ns, tid);
        __syncthreads();
        if (c0 + kGSlice < d) {
            qr.fetch(q_row, c0 + kGSlice, d, tid);
            nr.fetch(n_row, c0 + kGSlice, d, tid);
        }
        const int groups = min(kGSlice, d - c0 + 15) >> 4;
        const float* nb = Ns + (16 * w + l15) * kGSS + 4 * gq;
        const float* qa = Qs + l15 * kGSS + 4 * gq;
        for (int G = 0; G < groups; ++G) {    // all operand reads of a group first, then its MFMAs
            const float4 b = lds4(nb + 16 * G);
            float4 a[RB];
#pragma unroll
            for (int r = 0; r < RB; ++r) a[r] = lds4(qa + 16 * r * kGSS + 16 * G);
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] = mfma16g(a[r].x, b.x, acc[r]);
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] = mfma16g(a[r].y, b.y, acc[r]);
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] = mfma16g(a[r].z, b.z, acc[r]);
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] = mfma16g(a[r].w, b.w, acc[r]);
        }
        __syncthreads();
    }
    const int n = n0 + 16 * w + l15;
    float* Srow = S + (int64_t)tc.wgrow * g.rows_tile * Npad;
    if (n < N) {
#pragma unroll
        for (int r = 0; r < RB; ++r) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * r + 4 * gq + v;
                if (row < tc.nrows) Srow[((int64_t)bx * g.rows_tile + row) * kGNeg + 16 * w + l15] = acc[r][v];
            }
        }
    }
}

// ---- row statistics and weights ------------------------------------------------------------
// One workgroup (16 waves) per row tile, one wave per row at a time.  A row of at most 1024 scores
// is read once into registers (16 per lane), reduced, and written back as the weights W = dL/dS:
// exp(S - lse) for the softmax losses, w sigmoid(S) for the logistic loss, the indicator of
// margin - f + S > 0 for the margin loss, 0 in the padding up to Npad; a longer row is read from the cache-resident buffer once per pass instead.
// rowa = dL/df, loss_partial[tile] = sum over the tile's rows.
constexpr int kStatThreads = 1024;
constexpr int kStatRegs = 16;                 // scores of a row per lane on the register path
template <int LOSS>
__global__ void __launch_bounds__(kStatThreads)
k_gemm_rowstats(BatchGeom g, BucketParams bp, float* __restrict__ S, const float* __restrict__ fpos, int Npad,
                float* __restrict__ rowa, double* __restrict__ loss_partial) {
    constexpr int WAVES = kStatThreads / kWave;
    __shared__ double wave_loss[WAVES];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const TileCoord tc = tile_coord(g, blockIdx.x);
    const int N = g.N;
    float* Stile = S + (int64_t)tc.wgrow * g.rows_tile * Npad;
    const bool in_regs = Npad <= kStatRegs * kWave;
    double loss = 0.0;
    for (int row = w; row < tc.nrows; row += WAVES) {
        float* s = Stile + (int64_t)row * kGNeg;          // element n of the row sits at s[(n / 64) * tstride + n % 64]
        const int64_t tstride = (int64_t)g.rows_tile * kGNeg;
        auto at = [&](int n) -> float& { return s[(n >> 6) * tstride + (n & 63)]; };
        const int64_t ridx = (int64_t)tc.si * g.P + tc.e0 + row;
        const float f = fpos[ridx];
        float x[kStatRegs];                               // x[j] = score lane + 64 j (register path)
        if (in_regs) {
#pragma unroll
            for (int j = 0; j < kStatRegs; ++j) x[j] = lane + kWave * j < N ? s[j * tstride + lane] : -INFINITY;
        }
        if (LOSS == LEGEND_LOSS_SOFTMAX) {
            float m = -INFINITY;
            if (in_regs) {
#pragma unroll
                for (int j = 0; j < kStatRegs; ++j) m = fmaxf(m, x[j]);
            } else {
                for (int n = lane; n < N; n += kWave) m = fmaxf(m, at(n));
            }
            for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
            if (bp.softmax_with_pos) m = fmaxf(m, f);
            float l = 0.f;
            if (in_regs) {
#pragma unroll
                for (int j = 0; j < kStatRegs; ++j) {     // same order of the lane's terms as the strided loop
                    if (lane + kWave * j < N) { x[j] = fast_exp(x[j] - m); l += x[j]; }
                }
            } else {
                for (int n = lane; n < N; n += kWave) l += fast_exp(at(n) - m);
            }
            for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off, kWave);
            float a = -1.f;
            if (bp.softmax_with_pos) {
                const float pf = expf(f - m);
                a = -l / (l + pf);            // minus the negatives' share of the sum: no cancellation where the positive dominates
                l += pf;
            }
            const float il = 1.f / l;
            if (in_regs) {
#pragma unroll
                for (int j = 0; j < kStatRegs; ++j) {
                    const int n = lane + kWave * j;
                    if (n < Npad) s[j * tstride + lane] = n < N ? x[j] * il : 0.f;
                }
            } else {
                for (int n = lane; n < Npad; n += kWave) at(n) = n < N ? fast_exp(at(n) - m) * il : 0.f;
            }
            if (lane == 0) rowa[ridx] = a;
            loss += (double)(m + logf(l) - f);
        } else if (LOSS == LEGEND_LOSS_MARGIN) {
            // pair (row, negative) pays margin - f + S where that is positive: W is the indicator, dL/df minus their count
            const float base = bp.margin - f;
            float t = 0.f, cnt = 0.f;
            if (in_regs) {
#pragma unroll
                for (int j = 0; j < kStatRegs; ++j) {
                    const int n = lane + kWave * j;
                    const float sh = n < N ? base + x[j] : 0.f;
                    const float wv = sh > 0.f ? 1.f : 0.f;
                    t += fmaxf(sh, 0.f);
                    cnt += wv;
                    if (n < Npad) s[j * tstride + lane] = wv;
                }
            } else {
                for (int n = lane; n < Npad; n += kWave) {
                    const float sh = n < N ? base + at(n) : 0.f;
                    const float wv = sh > 0.f ? 1.f : 0.f;
                    t += fmaxf(sh, 0.f);
                    cnt += wv;
                    at(n) = wv;
                }
            }
            for (int off = 32; off > 0; off >>= 1) { t += __shfl_xor(t, off, kWave); cnt += __shfl_xor(cnt, off, kWave); }
            if (lane == 0) rowa[ridx] = -cnt;
            loss += (double)t;
        } else {
            float t = 0.f;
            if (in_regs) {
#pragma unroll
                for (int j = 0; j < kStatRegs; ++j) {
                    const int n = lane + kWave * j;
                    if (n < N) t += softplusf(x[j]);
                    if (n < Npad) s[j * tstride + lane] = n < N ? bp.neg_weight * sigmoidf(x[j]) : 0.f;
                }
            } else {
                for (int n = lane; n < N; n += kWave) t += softplusf(at(n));
            }
            for (int off = 32; off > 0; off >>= 1) t += __shfl_xor(t, off, kWave);
            if (!in_regs)
                for (int n = lane; n < Npad; n += kWave) at(n) = n < N ? bp.neg_weight * sigmoidf(at(n)) : 0.f;
            if (lane == 0) rowa[ridx] = -sigmoidf(-f);
            loss += (double)(softplusf(-f) + bp.neg_weight * t);
        }
    }
    if (lane == 0) wave_loss[w] = loss;
    __syncthreads();
    if (tid == 0) {
        double t = 0.0;
        for (int k = 0; k < WAVES; ++k) t += wave_loss[k];
        loss_partial[blockIdx.x] = t;
    }
}

// ---- G_Q = W Neg ---------------------------------------------------------------------------------
// grid: (column tiles of CT, row tiles).  CT / 16 waves; wave w owns columns 16w..16w+15 of the
// tile and all row blocks; the negatives are streamed 64 at a time, the next tile in flight.
// (A multiple of four waves keeps the four SIMDs of a compute unit evenly loaded between the
// workgroup barriers.)
constexpr int kGColTile = 128;            // G_Q: eight waves, 64 KB of LDS, two workgroups per compute unit
constexpr int kGNegColTile = 80;          // G_neg: five waves; a 128-column Q slice would leave room for one workgroup only (slower)
template <int CT, int RB>
__global__ void __launch_bounds__(CT * 4)
k_gemm_gq(BatchGeom g, BucketParams bp, const int32_t* __restrict__ neg_ids, const float* __restrict__ W, int Npad,
          float* __restrict__ GQ, int nx, int64_t ny) {
    constexpr int THREADS = CT * 4, CS = CT + 4;
    extern __shared__ __align__(16) float gq_smem[];
    float* Wt = gq_smem;                      // [112][68]
    float* Nt = Wt + kGRows * kGWS;           // [64][CT + 4]
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l15 = lane & 15, gq = lane >> 4;
    int bx;
    int64_t by;
    if (!xcd_tile((int64_t)nx * ny, nx, &bx, &by)) return;       // uniform
    const TileCoord tc = tile_coord(g, by);
    const int c0 = bx * CT;
    const int N = g.N, d = bp.dim;
    const float* En = tc.side == 0 ? bp.E_dst : bp.E_src;
    const int32_t* my_negs = neg_ids + ((int64_t)tc.si * g.nchunks + tc.c) * N;
    const float* Wtile = W + (int64_t)tc.wgrow * g.rows_tile * Npad;

    WTileRegs<THREADS> wr;
    SliceRegs<THREADS, kGNeg, CT> nr;
    auto neg_row = [&](int n0) {
        return [=](int row) -> const float* { return n0 + row < N ? En + (int64_t)my_negs[n0 + row] * d : nullptr; };
    };
    wr.fetch(Wtile, g.rows_tile, tc.nrows, 0, tid);
    nr.fetch(neg_row(0), c0, d, tid);

    f32x4 acc[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int n0 = 0; n0 < N; n0 += kGNeg) {
        wr.store(Wt, tid);
        nr.store(Nt, tid);
        __syncthreads();
        if (n0 + kGNeg < N) {
            wr.fetch(Wtile, g.rows_tile, tc.nrows, n0 + kGNeg, tid);
            nr.fetch(neg_row(n0 + kGNeg), c0, d, tid);
        }
        const int groups = c0 + 16 * w < d ? (min(kGNeg, N - n0) + 15) >> 4 : 0;    // nothing for a column block past d
        const float* wa = Wt + l15 * kGWS + 4 * gq;
        const float* nb = Nt + (4 * gq) * CS + 16 * w + l15;
        for (int G = 0; G < groups; ++G) {
            float b[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) b[s] = nb[(16 * G + s) * CS];
            float4 a[RB];
#pragma unroll
            for (int r = 0; r < RB; ++r) a[r] = lds4(wa + 16 * r * kGWS + 16 * G);
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] = mfma16g(a[r].x, b[0], acc[r]);
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] = mfma16g(a[r].y, b[1], acc[r]);
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] = mfma16g(a[r].z, b[2], acc[r]);
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] = mfma16g(a[r].w, b[3], acc[r]);
        }
        __syncthreads();
    }
    const int col = c0 + 16 * w + l15;
    if (col < d) {
        float* out = GQ + ((int64_t)tc.si * g.P + tc.e0) * d + col;
#pragma unroll
        for (int r = 0; r < RB; ++r) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * r + 4 * gq + v;
                if (row < tc.nrows) out[(int64_t)row * d] = acc[r][v];
            }
        }
    }
}

// ---- G_neg = W^T Q -------------------------------------------------------------------------------
// grid: (column tiles of CT, row tiles).  The Q slice of the column tile stays in LDS; the
// negatives are walked 64 at a time; wave w owns columns 16w..16w+15 and the four 16-negative
// blocks of a tile.  Both operands have the contraction index (the row) as the slow one.
template <int CT>
__global__ void __launch_bounds__(CT * 4)
k_gemm_gneg(BatchGeom g, BucketParams bp, const int32_t* __restrict__ neg_ids, const float* __restrict__ W, int Npad,
            const float* __restrict__ Q, float* __restrict__ grad, int nx, int64_t ny) {
    extern __shared__ __align__(16) float gneg_smem[];
    constexpr int THREADS = CT * 4, CS = CT + 4;
    float* Wt = gneg_smem;                    // [112][68]
    float* Qs = Wt + kGRows * kGWS;           // [112][CT + 4]
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, l15 = lane & 15, gq = lane >> 4;
    int bx;
    int64_t by;
    if (!xcd_tile((int64_t)nx * ny, nx, &bx, &by)) return;       // uniform
    const TileCoord tc = tile_coord(g, by);
    const int c0 = bx * CT;
    const int N = g.N, d = bp.dim;
    const int32_t* my_negs = neg_ids + ((int64_t)tc.si * g.nchunks + tc.c) * N;
    const float* Wtile = W + (int64_t)tc.wgrow * g.rows_tile * Npad;
    const float* Qrows = Q + ((int64_t)tc.si * g.P + tc.e0) * d;
    const int kgroups = (tc.nrows + 15) >> 4;
    const bool atomic = bp.atomic_mode != 0;
    float* Gn = tc.side == 0 ? bp.G_dst : bp.G_src;
    const int64_t neg_base = (int64_t)tc.si * g.per_side + (int64_t)g.roles * g.P + ((int64_t)tc.c * g.T + tc.t_row) * N;

    WTileRegs<THREADS> wr;
    wr.fetch(Wtile, g.rows_tile, tc.nrows, 0, tid);
    {
        SliceRegs<THREADS, kGRows, CT> qr;
        const int nrows = tc.nrows;
        qr.fetch([=](int row) -> const float* { return row < nrows ? Qrows + (int64_t)row * d : nullptr; }, c0, d, tid);
        qr.store(Qs, tid);
    }
    const int col = c0 + 16 * w + l15;
    const bool col0_live = c0 + 16 * w < d;   // uniform per wave
    for (int n0 = 0; n0 < N; n0 += kGNeg) {
        __syncthreads();                      // the previous tile's W has been consumed
        wr.store(Wt, tid);
        __syncthreads();
        if (n0 + kGNeg < N) wr.fetch(Wtile, g.rows_tile, tc.nrows, n0 + kGNeg, tid);
        f32x4 acc[4];
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) acc[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
        const float* wa = Wt + (4 * gq) * kGWS + l15;
        const float* qb = Qs + (4 * gq) * CS + 16 * w + l15;
        for (int G = 0; G < (col0_live ? kgroups : 0); ++G) {    // all operand reads of a group first, then its MFMAs
            float b[4], a[4][4];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                b[s] = qb[(16 * G + s) * CS];
#pragma unroll
                for (int mb = 0; mb < 4; ++mb) a[s][mb] = wa[(16 * G + s) * kGWS + 16 * mb];
            }
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int mb = 0; mb < 4; ++mb) acc[mb] = mfma16g(a[s][mb], b[s], acc[mb]);
        }
        if (col < d) {
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int n = n0 + 16 * mb + 4 * gq + v;
                    if (n < N) {
                        if (atomic) unsafeAtomicAdd(Gn + (int64_t)my_negs[n] * d + col, acc[mb][v]);
                        else grad[(neg_base + n) * d + col] = acc[mb][v];
                    }
                }
            }
        }
    }
}

// ---- chain rule for the positives ---------------------------------------------------------------
template <int SCORE>
__global__ void __launch_bounds__(128)
k_gemm_chain(BatchGeom g, BucketParams bp, const float* __restrict__ Q, const float* __restrict__ GQ,
             const float* __restrict__ rowa, float* __restrict__ grad) {
    const int64_t idx = blockIdx.x;
    const int si = (int)(idx / g.P);
    const int64_t e = idx % g.P;
    const int side = g.side_id[si];
    const int d = bp.dim;
    const int32_t* eb = bp.edges + (bp.batch_lo + e) * 3;
    const int xid = eb[side == 0 ? 0 : 2], yid = eb[side == 0 ? 2 : 0], rid = eb[1];
    const float* x = (side == 0 ? bp.E_src : bp.E_dst) + (int64_t)xid * d;
    const float* y = (side == 0 ? bp.E_dst : bp.E_src) + (int64_t)yid * d;
    const float* r = SCORE == LEGEND_SCORE_DOT ? x : bp.E_rel + (int64_t)rid * d;
    const float* q = Q + idx * d;
    const float* gqr = GQ + idx * d;
    const float a = rowa[idx];
    const bool atomic = bp.atomic_mode != 0;
    const int64_t side_base = (int64_t)si * g.per_side;
    float* gx = grad + (side_base + (side == 0 ? 0 : g.P) + e) * d;
    float* gy = grad + (side_base + (side == 0 ? g.P : 0) + e) * d;
    float* gr = grad + (side_base + 2 * (int64_t)g.P + e) * d;
    if (atomic) {
        gx = (side == 0 ? bp.G_src : bp.G_dst) + (int64_t)xid * d;
        gy = (side == 0 ? bp.G_dst : bp.G_src) + (int64_t)yid * d;
        gr = bp.G_rel + (int64_t)rid * d;
    }
    auto emit = [&](float* p, float v) {
        if (atomic) unsafeAtomicAdd(p, v);
        else *p = v;
    };
    if (SCORE == LEGEND_SCORE_COMPLEX) {
        const int h = d >> 1;
        for (int k = threadIdx.x; k < h; k += 128) {
            const float xr = x[k], xi = x[k + h], rr = r[k], ri = r[k + h];
            const float gre = gqr[k] + a * y[k], gim = gqr[k + h] + a * y[k + h];
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
        for (int k = threadIdx.x; k < d; k += 128) {
            const float gv = gqr[k] + a * y[k];
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

int64_t gemm_npad(int N) { return ((int64_t)N + kGNeg - 1) / kGNeg * kGNeg; }

hipError_t launch_chunks_gemm(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    if (bp.dim <= kNarrowMaxDim || bp.dim > kWideMaxDim || g.rows_tile > kGRows || !ws.gemm_Q)
        return hipErrorInvalidValue;
    const int64_t tiles = (int64_t)g.sides * g.nchunks * g.T;
    const int64_t rows = (int64_t)g.sides * g.P;
    const int Npad = (int)gemm_npad(g.N);
    const int ntiles = Npad / kGNeg;
    const int coltiles = (bp.dim + kGColTile - 1) / kGColTile;
    const bool softmax = bp.loss == LEGEND_LOSS_SOFTMAX;
    const int negtiles = (bp.dim + kGNegColTile - 1) / kGNegColTile;
    const size_t gneg_lds = sizeof(float) * (kGRows * kGWS + kGRows * (kGNegColTile + 4));
    const size_t gq_lds = sizeof(float) * (kGRows * kGWS + kGNeg * (kGColTile + 4));
    static PerDeviceFlag configured;
    if (configured.pending()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_gneg<kGNegColTile>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)gneg_lds);
        if (e != hipSuccess) return e;
        configured.set();
    }
    switch (bp.score) {
        case LEGEND_SCORE_DOT:
            hipLaunchKernelGGL(k_gemm_compose<LEGEND_SCORE_DOT>, dim3((unsigned)rows), dim3(128), 0, st, g, bp, ws.gemm_Q, ws.gemm_f);
            break;
        case LEGEND_SCORE_DISTMULT:
            hipLaunchKernelGGL(k_gemm_compose<LEGEND_SCORE_DISTMULT>, dim3((unsigned)rows), dim3(128), 0, st, g, bp, ws.gemm_Q, ws.gemm_f);
            break;
        default:
            hipLaunchKernelGGL(k_gemm_compose<LEGEND_SCORE_COMPLEX>, dim3((unsigned)rows), dim3(128), 0, st, g, bp, ws.gemm_Q, ws.gemm_f);
            break;
    }
    const int rb = (g.rows_tile + 15) / 16;
#define LEGEND_GEMM_RB(RB)                                                                                             \
    case RB:                                                                                                           \
        hipLaunchKernelGGL(k_gemm_scores<RB>, dim3((unsigned)xcd_grid(ntiles * tiles)), dim3(256), 0, st, g, bp, ws.neg_ids, \
                           ws.gemm_Q, ws.gemm_S, Npad, ntiles, tiles);                                                 \
        break;
    switch (rb) {
        LEGEND_GEMM_RB(1) LEGEND_GEMM_RB(2) LEGEND_GEMM_RB(3) LEGEND_GEMM_RB(4) LEGEND_GEMM_RB(5) LEGEND_GEMM_RB(6)
        default: hipLaunchKernelGGL(k_gemm_scores<7>, dim3((unsigned)xcd_grid(ntiles * tiles)), dim3(256), 0, st, g, bp,
                                    ws.neg_ids, ws.gemm_Q, ws.gemm_S, Npad, ntiles, tiles);
    }
#undef LEGEND_GEMM_RB
    if (softmax)
        hipLaunchKernelGGL(k_gemm_rowstats<LEGEND_LOSS_SOFTMAX>, dim3((unsigned)tiles), dim3(kStatThreads), 0, st, g, bp,
                           ws.gemm_S, ws.gemm_f, Npad, ws.gemm_a, ws.loss_partial);
    else if (bp.loss == LEGEND_LOSS_MARGIN)
        hipLaunchKernelGGL(k_gemm_rowstats<LEGEND_LOSS_MARGIN>, dim3((unsigned)tiles), dim3(kStatThreads), 0, st, g, bp,
                           ws.gemm_S, ws.gemm_f, Npad, ws.gemm_a, ws.loss_partial);
    else
        hipLaunchKernelGGL(k_gemm_rowstats<LEGEND_LOSS_LOGISTIC>, dim3((unsigned)tiles), dim3(kStatThreads), 0, st, g, bp,
                           ws.gemm_S, ws.gemm_f, Npad, ws.gemm_a, ws.loss_partial);
#define LEGEND_GEMM_RB(RB)                                                                                             \
    case RB: {                                                                                                         \
        static PerDeviceFlag gq_configured;                                                                            \
        if (gq_configured.pending()) {                                                                                 \
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_gq<kGColTile, RB>),                         \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)gq_lds);                          \
            if (e != hipSuccess) return e;                                                                             \
            gq_configured.set();                                                                                       \
        }                                                                                                              \
        hipLaunchKernelGGL((k_gemm_gq<kGColTile, RB>), dim3((unsigned)xcd_grid(coltiles * tiles)), dim3(kGColTile * 4), gq_lds, \
                           st, g, bp, ws.neg_ids, ws.gemm_S, Npad, ws.gemm_G, coltiles, tiles);                        \
        break;                                                                                                         \
    }
    {
        hipError_t e = hipSuccess;
        switch (rb < 7 ? rb : 7) {
            LEGEND_GEMM_RB(1) LEGEND_GEMM_RB(2) LEGEND_GEMM_RB(3) LEGEND_GEMM_RB(4) LEGEND_GEMM_RB(5) LEGEND_GEMM_RB(6)
            LEGEND_GEMM_RB(7)
        }
    }
#undef LEGEND_GEMM_RB
    hipLaunchKernelGGL(k_gemm_gneg<kGNegColTile>, dim3((unsigned)xcd_grid(negtiles * tiles)), dim3(kGNegColTile * 4), gneg_lds, st, g,
                       bp, ws.neg_ids, ws.gemm_S, Npad, ws.gemm_Q, ws.grad, negtiles, tiles);
    switch (bp.score) {
        case LEGEND_SCORE_DOT:
            hipLaunchKernelGGL(k_gemm_chain<LEGEND_SCORE_DOT>, dim3((unsigned)rows), dim3(128), 0, st, g, bp, ws.gemm_Q, ws.gemm_G, ws.gemm_a, ws.grad);
            break;
        case LEGEND_SCORE_DISTMULT:
            hipLaunchKernelGGL(k_gemm_chain<LEGEND_SCORE_DISTMULT>, dim3((unsigned)rows), dim3(128), 0, st, g, bp, ws.gemm_Q, ws.gemm_G, ws.gemm_a, ws.grad);
            break;
        default:
            hipLaunchKernelGGL(k_gemm_chain<LEGEND_SCORE_COMPLEX>, dim3((unsigned)rows), dim3(128), 0, st, g, bp, ws.gemm_Q, ws.gemm_G, ws.gemm_a, ws.grad);
            break;
    }
    return hipGetLastError();
}

}  // namespace legend
