// Single-sweep batch computation for the paper's large workloads: Eq. 1 loss, dim = 100 (also 64), at most
// 1024 negatives per chunk (paper Sec. 2.1 stage 5, Sec. 6).  The general kernel reads the
// chunk's negatives twice because the row log-sum-exp must be known before any gradient.  Here
// the softmax numerators are taken against a reference m_e fixed after the first tile of
// negatives, the row maximum over that tile (the tiles interleave the chunk's negatives, so the
// first one is an even sample of them):
//     P_en = c exp(S_en - m_e),   l_e = sum_n P_en,   W_en = P_en / l_e,   loss_e = m_e + log(l_e / c) - f_e,
// (c = 2^-58 makes room for scores above m_e),
// so one sweep over the negatives yields the unnormalised G_Q = sum_n P_en theta_n, and the P
// blocks (64 x N values, the paper's "Intermediate Result 3") stay in the register file of the
// workgroup: eight waves, 128 registers per lane each, one workgroup per compute unit.  After
// the sweep the stored numerators are scaled by 1 / l_e and G_neg = W^T Q is formed straight from
// the stored blocks.  The reference is rescaled by exception (the online form of the softmax, paid
// for only where it is needed): a wave whose 16 negatives of a tile hold a score more than a limit
// (110 unless overridden; the numerators stay far from overflow) above the row's current reference
// takes its own row maxima as the reference for its share of that tile and says so in LDS; the waves
// that add the tile to G_Q bring every share to a common new reference (factors exp(ref - new) <= 1
// on the W operands and on their accumulators) and publish it for the group's next tile.  Every
// wave's reference per tile is kept in LDS, and after the sweep the stored numerators and both
// groups' accumulators are brought to the final reference, the largest of all.  Nothing is ever
// computed twice.  Only a row sum that is not finite makes the workgroup write nothing and flag
// itself; the general two-sweep kernel then redoes the chunk.
//
// Work split (16x16x4 fp32 MFMA; g = lane / 16, l15 = lane % 16).  The eight waves form two
// groups of four; the negatives are dealt into tiles of 64 (negative n sits in tile n mod T),
// even tiles for group 0, odd ones for group 1; wave wl of a group:
//   sweep, per tile of its group:
//     scores    owns the 16 negatives 16wl..16wl+15 of the tile, which it has gathered itself,
//               and all 64 rows: four 16x16 blocks S[16r + 4g + v][16wl + l15], r, v = 0..3;
//     P         the same 16 values per lane, kept for the whole kernel, and written to LDS as
//               W[row][negative] for the next step;
//     G_Q       adds W[16wl..16wl+15, tile] x Neg[tile, :] to its 16 x 112 slice; the partial
//               sums of the two groups are added once at the end;
//   the two groups run half a step apart, so that one is in the vector-ALU part of its step
//   while the other keeps the matrix pipe busy;
//   afterwards, per tile and with no workgroup barrier:
//     G_neg     contracts its stored P (as the A operand of P^T: lane = negative, k = row)
//               with Q^T read from LDS over all 64 rows, stages its 16 gradient rows in
//               its own LDS area and writes them out as whole rows of 16-byte pieces.
#include <type_traits>

#include "chunk_common.h"

#ifndef LEGEND_FAST_SCORE
#define LEGEND_FAST_SCORE 0     // 0 Dot (and the dispatch), 1 DistMult, 2 ComplEx: one translation unit each
#endif

namespace legend {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x4 mfma16(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// compile-time loop: the body gets its index as an integral constant, so arrays indexed by it
// are scalarised into registers
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr int kFThreads = 512;
constexpr int kFWaves = kFThreads / kWave;
constexpr int kFRow = 64;                // rows of Q per workgroup
constexpr int kFTile = 64;               // negatives per tile of a wave group: 16 per wave
constexpr int kFWS = kFTile + 4;         // row stride of a W tile
constexpr int kFQT = kFRow + 4;          // row stride of the transposed, scaled Q
constexpr int kFMaxSteps = 8;            // tiles per wave group: 1024 negatives in all
// The numerators are kept as exp(S - m) * 2^-58, m the row maximum of the first tile: scores up
// to `limit` (110) above m still give numerators far from overflow, and what lies more than
// about 47 below m would have a weight under 1e-20 anyway.  The factor is applied inside the
// exponential (below), not by moving m: S - m must keep its full precision.
constexpr float kFLiftLn = 58.f * 0.693147180559945309f;

// exp(x) * 2^-58 for x <= 110 without overflow: 2^(h/2) is scaled by 2^-29 and squared.
__device__ inline float fast_exp_lifted(float x) {
    const float L2E_HI = 1.44269502162933349609375f;
    const float L2E_LO = 1.925963033500011e-8f;
    const float hi = x * L2E_HI;
    float lo = fmaf(x, L2E_HI, -hi);
    lo = fmaf(x, L2E_LO, lo);
    const float r = __builtin_amdgcn_exp2f(0.5f * hi) * 1.862645149230957e-9f;     // 2^-29
    const float r2 = r * r;
    return fmaf(r2, lo * 0.6931471805599453f, r2);
}

template <int D>
struct FastShape {
    static_assert(D % 4 == 0 && D <= 112, "dimension must be a multiple of 4, at most 112");
    static constexpr int QS = ((D + 7) & ~7) + 4;          // row stride of Q and of the negatives tile
    static constexpr int KG = D / 16;                       // full groups of 16 along the dimension
    static constexpr int KT = (D % 16) / 4;                 // single steps of 4 after them
    static constexpr int NJ = (D + 15) / 16;                // 16-column blocks of a gradient row
    // Columns of the G_Q accumulator blocks (B operand and result column of lane l15 in block j), chosen so
    // that a lane's B operands of several blocks are adjacent in a row of the negatives tile:
    //   N4 groups of four blocks, block 4q + t holds column 64q + 4 l15 + t (one 128-bit LDS read per group),
    //   then N2 (0 or 1) pair of blocks, block t of it holds column 64 N4 + 2 l15 + t (one 64-bit read),
    //   then N1 single blocks holding column 64 N4 + 32 N2 + 16 q + l15.
    static constexpr int N4 = D / 64;
    static constexpr int N2 = (D - 64 * N4) / 32;
    static constexpr int N1 = (D - 64 * N4 - 32 * N2 + 15) / 16;
    static_assert(4 * N4 + 2 * N2 + N1 == NJ, "column blocks");
    static constexpr int LPR = 32;                          // lanes per gathered row (float4 each)
    static constexpr int STEPS = 16 / (kWave / LPR);        // a wave gathers 16 rows, two at a time
    static constexpr int q_floats = kFRow * QS;
    static constexpr int n_floats = 2 * kFTile * QS + 16;   // one tile per wave group; + slack: column blocks run past the last row
    static constexpr int w_floats = 2 * kFRow * kFWS > 16 * NJ * kFQT ? 2 * kFRow * kFWS : 16 * NJ * kFQT;
    static constexpr int r_floats = 2 * kFMaxSteps * 4 * kFRow;   // every wave's softmax reference per tile and row
    static constexpr size_t lds_bytes = sizeof(float) * (q_floats + n_floats + w_floats + 11 * kFRow + 48 + kIdsLds + r_floats);
};

// Four elements of an embedding row that are handled together: elements 4c..4c+3, or for
// ComplEx the real and imaginary parts of the complex components 2c and 2c+1 (elements 2c,
// 2c+1, D/2+2c, D/2+2c+1; paper Sec. 2.1, score functions of Table 1).
template <int SCORE, int D>
struct RowItem {
    static constexpr int H = D / 2;
    static_assert(SCORE != LEGEND_SCORE_COMPLEX || H % 2 == 0, "ComplEx items need an even number of components");
    __device__ static void load(const float* row, int c, float (&v)[4]) {
        if (SCORE == LEGEND_SCORE_COMPLEX) {
            const float2 a = *reinterpret_cast<const float2*>(row + 2 * c);
            const float2 b = *reinterpret_cast<const float2*>(row + H + 2 * c);
            v[0] = a.x; v[1] = a.y; v[2] = b.x; v[3] = b.y;
        } else {
            const float4 a = *reinterpret_cast<const float4*>(row + 4 * c);
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        }
    }
    __device__ static void store(float* row, int c, const float (&v)[4]) {
        if (SCORE == LEGEND_SCORE_COMPLEX) {
            *reinterpret_cast<float2*>(row + 2 * c) = make_float2(v[0], v[1]);
            *reinterpret_cast<float2*>(row + H + 2 * c) = make_float2(v[2], v[3]);
        } else {
            *reinterpret_cast<float4*>(row + 4 * c) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
    // q = x (.) r for the destination side, conj(r) (.) x for the source side
    __device__ static void compose(int side, const float (&x)[4], const float (&r)[4], float (&q)[4]) {
        if (SCORE == LEGEND_SCORE_DOT) {
#pragma unroll
            for (int t = 0; t < 4; ++t) q[t] = x[t];
        } else if (SCORE == LEGEND_SCORE_DISTMULT) {
#pragma unroll
            for (int t = 0; t < 4; ++t) q[t] = x[t] * r[t];
        } else {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const float xr = x[p], xi = x[p + 2], rr = r[p], ri = r[p + 2];
                if (side == 0) { q[p] = xr * rr - xi * ri; q[p + 2] = xr * ri + xi * rr; }
                else           { q[p] = rr * xr + ri * xi; q[p + 2] = rr * xi - ri * xr; }
            }
        }
    }
    // gradients of x and r from the gradient of q
    __device__ static void chain(int side, const float (&x)[4], const float (&r)[4], const float (&gq)[4],
                                 float (&gx)[4], float (&gr)[4]) {
        if (SCORE == LEGEND_SCORE_DOT) {
#pragma unroll
            for (int t = 0; t < 4; ++t) { gx[t] = gq[t]; gr[t] = 0.f; }
        } else if (SCORE == LEGEND_SCORE_DISTMULT) {
#pragma unroll
            for (int t = 0; t < 4; ++t) { gx[t] = r[t] * gq[t]; gr[t] = x[t] * gq[t]; }
        } else {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const float xr = x[p], xi = x[p + 2], rr = r[p], ri = r[p + 2];
                const float gre = gq[p], gim = gq[p + 2];
                if (side == 0) {
                    gx[p] = rr * gre + ri * gim;      gx[p + 2] = rr * gim - ri * gre;
                    gr[p] = xr * gre + xi * gim;      gr[p + 2] = xr * gim - xi * gre;
                } else {
                    gx[p] = rr * gre - ri * gim;      gx[p + 2] = rr * gim + ri * gre;
                    gr[p] = gre * xr + gim * xi;      gr[p + 2] = gre * xi - gim * xr;
                }
            }
        }
    }
};

template <int SCORE, int D>
__global__ void __launch_bounds__(kFThreads, 1)
k_chunk_fast(BatchGeom g, BucketParams bp, const int32_t* __restrict__ neg_ids, float* __restrict__ grad,
             double* __restrict__ loss_partial, uint32_t* __restrict__ redo, unsigned long long* __restrict__ redo_total,
             float limit, int rescale_allowed) {
    using Sh = FastShape<D>;
    using Item = RowItem<SCORE, D>;
    constexpr int QS = Sh::QS, KG = Sh::KG, KT = Sh::KT, NJ = Sh::NJ, STEPS = Sh::STEPS;
    constexpr int N4 = Sh::N4, N2 = Sh::N2, N1 = Sh::N1;
    constexpr int d = D;

    extern __shared__ __align__(16) float smem[];
    float* Qs = smem;
    float* Ns = Qs + Sh::q_floats;
    float* Ws = Ns + Sh::n_floats;              // sweep: W[2][64][68]; before: partial f; afterwards: row sums, then Q^T [112][68]
    float* ref_s = Ws + Sh::w_floats;           // [64] softmax reference: row maximum over the first tile
    float* scale_s = ref_s + kFRow;             // [64] 1 / l_e
    float* logl_s = scale_s + kFRow;            // [64] log l_e
    float* rowloss_s = logl_s + kFRow;          // [64]
    float* f_s = rowloss_s + kFRow;             // [64] positive scores
    float* mx_s = f_s + kFRow;                  // [4][64] per-wave row maxima of the first tile
    float* Rtab = mx_s + 4 * kFRow;             // [2][64] reference of each wave group's G_Q accumulators
    uint32_t* flag_s = reinterpret_cast<uint32_t*>(Rtab + 2 * kFRow);    // [16]: 0..7 unused, 8 row sum not finite, 9 some reference was raised
    uint32_t* bump_s = flag_s + 16;             // [2][16]: a wave of the group raised its reference in this tile
    int32_t* ids_s = reinterpret_cast<int32_t*>(bump_s + 32);            // [kIdsLds]
    float* refw_s = reinterpret_cast<float*>(ids_s + kIdsLds);           // [2][kFMaxSteps][4][64]

    const int tid = threadIdx.x;
    const int w = tid >> 6;
    const int lane = tid & 63;
    const int l15 = lane & 15;
    const int gq = lane >> 4;                   // lane group: the k index a lane supplies to an MFMA

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

    for (int k = tid; k < N; k += kFThreads) ids_s[k] = my_negs[k];         // N <= 1024 here
    if (tid < 48) flag_s[tid] = 0;              // flags and the per-tile marks behind them

    // ---- prologue: Q rows and positive scores ---------------------------------------------------
    // A row is cut into D/4 items of four elements; a thread takes up to ITEMS (row, item) pairs
    // and issues all its loads before it uses any of them.
    constexpr int IPR = D / 4;
    constexpr int ITEMS = (kFRow * IPR + kFThreads - 1) / kFThreads;
    int it_row[ITEMS], it_c[ITEMS];
#pragma unroll
    for (int s = 0; s < ITEMS; ++s) {
        const int idx = tid + kFThreads * s;
        it_row[s] = idx / IPR;
        it_c[s] = idx - it_row[s] * IPR;
    }
    {
        float* part_s = Ws;                   // [64][IPR] partial positive scores
        int32_t ex[ITEMS], ey[ITEMS], er[ITEMS];
#pragma unroll
        for (int s = 0; s < ITEMS; ++s) {
            const bool live = it_row[s] < nrows;
            ex[s] = live ? eb[it_row[s] * 3 + xcol] : 0;
            ey[s] = live ? eb[it_row[s] * 3 + ycol] : 0;
            er[s] = live && SCORE != LEGEND_SCORE_DOT ? eb[it_row[s] * 3 + 1] : 0;
        }
        float x[ITEMS][4], y[ITEMS][4], r[ITEMS][4];
#pragma unroll
        for (int s = 0; s < ITEMS; ++s) {
            Item::load(Ex + (int64_t)ex[s] * d, it_c[s], x[s]);
            Item::load(Ey + (int64_t)ey[s] * d, it_c[s], y[s]);
            if (SCORE != LEGEND_SCORE_DOT) Item::load(bp.E_rel + (int64_t)er[s] * d, it_c[s], r[s]);
        }
#pragma unroll
        for (int s = 0; s < ITEMS; ++s) {
            if (it_row[s] < kFRow) {
                float q[4] = {0.f, 0.f, 0.f, 0.f};
                float partial = 0.f;
                if (it_row[s] < nrows) {
                    Item::compose(side, x[s], r[s], q);
#pragma unroll
                    for (int t = 0; t < 4; ++t) partial += q[t] * y[s][t];
                }
                Item::store(Qs + it_row[s] * QS, it_c[s], q);
                part_s[it_row[s] * IPR + it_c[s]] = partial;
            }
        }
        __syncthreads();
        if (tid < kFRow) {
            float f = 0.f;
            for (int cc = 0; cc < IPR; ++cc) f += part_s[tid * IPR + cc];
            f_s[tid] = f;
        }
    }

    // ---- gather machinery: a wave fetches rows 16wl..16wl+15 of its group's 64-negative tile -----
    const int grp = w >> 2, wl = w & 3;       // wave group and wave within it
    float* Ng = Ns + grp * (kFTile * QS);
    float* Wg = Ws + grp * (kFRow * kFWS);
    float4 pf[STEPS];
    // The lane's share of a gathered row is recomputed from the lane number wherever it is needed (two
    // instructions the compiler may not hoist): kept live across the kernel it ends up in scratch
    // memory, and its reload then sits in front of every tile's gather.
    auto lane_now = [&]() __attribute__((always_inline)) {
        int x;
        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(x));
        return x;
    };
    typedef __attribute__((address_space(3))) const int32_t* lds_ids_t;
    // Column k of tile t is negative k * ntiles + t: every tile is an even sample of the chunk's
    // negatives (uniform and degree-weighted ones alike), so the row maxima of the first tile
    // are a good reference for all of them.
    const int ntiles = (N + kFTile - 1) / kFTile;
    auto neg_of = [&](int t, int k) { return k * ntiles + t; };
    auto gather_issue = [&](int t) __attribute__((always_inline)) {
        const int ln = lane_now();
        const int grow_lane = ln >> 5;
        const int gcol_ld = (ln & 31) * 4 < d ? (ln & 31) * 4 : 0;
        int32_t idv[STEPS];
#pragma unroll
        for (int s = 0; s < STEPS; ++s) idv[s] = ((lds_ids_t)ids_s)[min(neg_of(t, wl * 16 + s * 2 + grow_lane), N - 1)];
#pragma unroll
        for (int s = 0; s < STEPS; ++s) pf[s] = *reinterpret_cast<const float4*>(En + (int64_t)idv[s] * d + gcol_ld);
    };
    auto gather_commit = [&](int t) __attribute__((always_inline)) {
        const int ln = lane_now();
        const int grow_lane = ln >> 5;
        const int gc0 = (ln & 31) * 4;
        if (neg_of(t, kFTile - 1) >= N) {     // columns past the last negative are zero rows
#pragma unroll
            for (int s = 0; s < STEPS; ++s)
                if (neg_of(t, wl * 16 + s * 2 + grow_lane) >= N) pf[s] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        if (gc0 < d) {
#pragma unroll
            for (int s = 0; s < STEPS; ++s)
                *reinterpret_cast<float4*>(Ng + (wl * 16 + s * 2 + grow_lane) * QS + gc0) = pf[s];
        }
    };

    // Tiles 2i belong to wave group 0 and tiles 2i + 1 to group 1.  The groups run half a step
    // apart: while one scores a tile and takes the exponentials (matrix pipe, then vector ALU
    // and LDS writes), the other multiplies its previous W tile into G_Q (matrix pipe with LDS
    // reads), so that the two waves of a SIMD want different units most of the time.
    auto tile_of = [&](int i) { return 2 * i + grp; };

    f32x4 P[kFMaxSteps][4];                   // the chunk's softmax numerators owned by this wave
    f32x4 accB[NJ];

    // scores of all 64 rows against the wave's own 16 negatives of its group's tile in LDS;
    // columns past the last negative get -1e30
    auto score_block = [&](int t, f32x4 (&acc)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
        const float* qa = Qs + l15 * QS + 4 * gq;
        const float* nb = Ng + (16 * wl + l15) * QS + 4 * gq;
#pragma unroll
        for (int G = 0; G < KG; ++G) {
            const float4 b = lds4(nb + 16 * G);
            float4 a[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) a[r] = lds4(qa + 16 * r * QS + 16 * G);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = mfma16(a[r].x, b.x, acc[r]);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = mfma16(a[r].y, b.y, acc[r]);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = mfma16(a[r].z, b.z, acc[r]);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = mfma16(a[r].w, b.w, acc[r]);
        }
#pragma unroll
        for (int ts = 0; ts < KT; ++ts) {
            const int k = 16 * KG + 4 * ts + gq;
            const float b = Ng[(16 * wl + l15) * QS + k];
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = mfma16(Qs[(16 * r + l15) * QS + k], b, acc[r]);
        }
        if (neg_of(t, 16 * wl + l15) >= N) {
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = f32x4{-1e30f, -1e30f, -1e30f, -1e30f};
        }
    };

    __syncthreads();                          // ids, Q and the positive scores are in LDS
#pragma unroll
    for (int j = 0; j < NJ; ++j) accB[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (tile_of(0) < ntiles) gather_issue(tile_of(0));
    float* Rg = Rtab + grp * kFRow;           // reference of this group's accumulators, per row
    // this wave's reference of tile i of its group, rows 0..63
    auto refw_of = [&](int g2, int i, int w2) { return refw_s + ((g2 * kFMaxSteps + i) * 4 + w2) * kFRow; };

    // scores and numerators of tile i of this group; P[i] is written
    // With FIRST (tile 0, wave group 0) the reference is made on the way: the row maxima of this
    // tile, exchanged between the four waves across one extra workgroup barrier.
    auto score_tile = [&](auto I, auto FIRST) __attribute__((always_inline)) {
        constexpr int i = decltype(I)::value;
        constexpr bool first = decltype(FIRST)::value;
        const int t = tile_of(i);
        gather_commit(t);                     // own rows only; their last readers are a barrier behind
        if (tile_of(i + 1) < ntiles) gather_issue(t + 2);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        f32x4 acc[4];
        score_block(t, acc);
        float4 reff[4];
        if (first) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float m = acc[r][v];
                    m = fmaxf(m, wave_shfl_xor(m, 1));
                    m = fmaxf(m, wave_shfl_xor(m, 2));
                    m = fmaxf(m, wave_shfl_xor(m, 4));
                    m = fmaxf(m, wave_shfl_xor(m, 8));
                    if (l15 == 0) mx_s[wl * kFRow + 16 * r + 4 * gq + v] = m;
                }
            }
            __syncthreads();                  // the other wave group passes the same barrier idle
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float4 m = lds4(mx_s + 16 * r + 4 * gq);
#pragma unroll
                for (int ww = 1; ww < 4; ++ww) {
                    const float4 o = lds4(mx_s + ww * kFRow + 16 * r + 4 * gq);
                    m.x = fmaxf(m.x, o.x); m.y = fmaxf(m.y, o.y); m.z = fmaxf(m.z, o.z); m.w = fmaxf(m.w, o.w);
                }
                // rows past the chunk: a huge reference turns every numerator into 0
                const int row = 16 * r + 4 * gq;
                m.x = row + 0 < nrows ? m.x : 1e30f;
                m.y = row + 1 < nrows ? m.y : 1e30f;
                m.z = row + 2 < nrows ? m.z : 1e30f;
                m.w = row + 3 < nrows ? m.w : 1e30f;
                reff[r] = m;
                if (wl == 0 && l15 == 0) {    // both groups' accumulators start at this reference
                    *reinterpret_cast<float4*>(Rtab + row) = m;
                    *reinterpret_cast<float4*>(Rtab + kFRow + row) = m;
                }
            }
        }
        // where this wave's reference of the tile is read from: the group's, or its own once raised
        const float* refp = Rg;
        float* own = refw_of(grp, i, wl);
        if (first) {
            if (l15 == 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) *reinterpret_cast<float4*>(own + 16 * r + 4 * gq) = reff[r];
            }
        } else {
            // a score beyond the reference by more than the limit: this wave goes on with its own row
            // maxima as the reference of its 16 negatives (never below the common one)
            float over = -1e30f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float4 rf = lds4(Rg + 16 * r + 4 * gq);
                over = fmaxf(over, fmaxf(fmaxf(acc[r][0] - rf.x, acc[r][1] - rf.y), fmaxf(acc[r][2] - rf.z, acc[r][3] - rf.w)));
                if (l15 == 0) *reinterpret_cast<float4*>(own + 16 * r + 4 * gq) = rf;
            }
            if (__builtin_expect(__ballot(over > limit) != 0ull, 0)) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float4 rf = lds4(Rg + 16 * r + 4 * gq);
                    float mm[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float m = acc[r][v];
                        m = fmaxf(m, wave_shfl_xor(m, 1));
                        m = fmaxf(m, wave_shfl_xor(m, 2));
                        m = fmaxf(m, wave_shfl_xor(m, 4));
                        m = fmaxf(m, wave_shfl_xor(m, 8));
                        mm[v] = m;
                    }
                    rf.x = fmaxf(rf.x, mm[0]); rf.y = fmaxf(rf.y, mm[1]); rf.z = fmaxf(rf.z, mm[2]); rf.w = fmaxf(rf.w, mm[3]);
                    if (l15 == 0) *reinterpret_cast<float4*>(own + 16 * r + 4 * gq) = rf;
                }
                if (lane == 0) {
                    bump_s[grp * 16 + i] = 1u;
                    flag_s[9] = 1u;
                    if (!rescale_allowed) flag_s[8] = 1u;      // test knob: hand the chunk to the two-sweep kernel instead
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                refp = own;
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float4 rf = first ? reff[r] : lds4(refp + 16 * r + 4 * gq);
            const float refv[4] = {rf.x, rf.y, rf.z, rf.w};
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float p = fast_exp_lifted(acc[r][v] - refv[v]);
                acc[r][v] = p;
                Wg[(16 * r + 4 * gq + v) * kFWS + 16 * wl + l15] = p;
            }
            P[i][r] = acc[r];
        }
    };
    // G_Q += W tile x negatives tile of this group: wave wl has rows 16wl..16wl+15, all columns
    auto accumulate_tile = [&](auto I) __attribute__((always_inline)) {
        constexpr int i = decltype(I)::value;
        const int t = tile_of(i);
        const float* wa = Wg + (16 * wl + l15) * kFWS + 4 * gq;
        // the four waves' shares of W are brought to one reference where a wave raised its own in this tile
        const bool bumped = bump_s[grp * 16 + i] != 0u;      // uniform
        const int arow = 16 * wl + l15;       // the row of this lane's A operands
        if (__builtin_expect(bumped, 0)) {
            float rnew = Rg[arow];
#pragma unroll
            for (int G = 0; G < 4; ++G) rnew = fmaxf(rnew, refw_of(grp, i, G)[arow]);
            // the accumulators (rows 16wl + 4g + v) follow the reference
            float4 ro = lds4(Rg + 16 * wl + 4 * gq), rn = ro;
#pragma unroll
            for (int G = 0; G < 4; ++G) {
                const float4 o = lds4(refw_of(grp, i, G) + 16 * wl + 4 * gq);
                rn.x = fmaxf(rn.x, o.x); rn.y = fmaxf(rn.y, o.y); rn.z = fmaxf(rn.z, o.z); rn.w = fmaxf(rn.w, o.w);
            }
            const f32x4 down = f32x4{fast_exp(ro.x - rn.x), fast_exp(ro.y - rn.y), fast_exp(ro.z - rn.z), fast_exp(ro.w - rn.w)};
#pragma unroll
            for (int j = 0; j < NJ; ++j) accB[j] *= down;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();  // every lane has read the old reference of the wave's rows
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (gq == 0) Rg[arow] = rnew;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
#pragma unroll
        for (int G = 0; G < 4; ++G) {
            if (neg_of(t, 16 * G) < N) {      // uniform: the group has a live column
                float4 a4 = lds4(wa + 16 * G);
                if (__builtin_expect(bumped, 0)) {
                    const float f = fast_exp(refw_of(grp, i, G)[arow] - Rg[arow]);     // <= 1
                    a4.x *= f; a4.y *= f; a4.z *= f; a4.w *= f;
                }
                const float av[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    // row k = 16G + 4g + s of the negatives tile; this lane's columns of it (gq_col)
                    const float* nrow = Ng + (16 * G + 4 * gq + s) * QS;
                    float b[NJ];
#pragma unroll
                    for (int q4 = 0; q4 < N4; ++q4) {
                        const float4 x = lds4(nrow + 64 * q4 + 4 * l15);
                        b[4 * q4] = x.x; b[4 * q4 + 1] = x.y; b[4 * q4 + 2] = x.z; b[4 * q4 + 3] = x.w;
                    }
                    if constexpr (N2 == 1) {
                        const float2 x = *reinterpret_cast<const float2*>(nrow + 64 * N4 + 2 * l15);
                        b[4 * N4] = x.x; b[4 * N4 + 1] = x.y;
                    }
#pragma unroll
                    for (int q1 = 0; q1 < N1; ++q1) b[4 * N4 + 2 * N2 + q1] = nrow[64 * N4 + 32 * N2 + 16 * q1 + l15];
#pragma unroll
                    for (int j = 0; j < NJ; ++j) accB[j] = mfma16(av[s], b[j], accB[j]);
                }
            }
        }
    };

    // ---- the sweep ---------------------------------------------------------------------------------
    // half-step h: group 0 scores tile h/2 (h even) or accumulates it (h odd); group 1 does the
    // same one half-step later.  Every branch below is uniform per wave, and the barrier count
    // depends on the tile count only.
    static_for<0, 2 * kFMaxSteps + 1>([&](auto Hh) {
        constexpr int h = decltype(Hh)::value;
        if (h <= ntiles) {
            if constexpr (h % 2 == 0) {
                if (grp == 0) {
                    if constexpr (h / 2 < kFMaxSteps) {
                        if (tile_of(h / 2) < ntiles)
                            score_tile(std::integral_constant<int, h / 2>{}, std::integral_constant<bool, h == 0>{});
                    }
                } else {
                    if constexpr (h == 0) __syncthreads();            // the barrier inside group 0's first tile
                    if constexpr (h >= 2) {
                        if (tile_of(h / 2 - 1) < ntiles) accumulate_tile(std::integral_constant<int, h / 2 - 1>{});
                    }
                }
            } else {
                if (grp == 0) {
                    if (tile_of(h / 2) < ntiles) accumulate_tile(std::integral_constant<int, h / 2>{});
                } else {
                    if (tile_of(h / 2) < ntiles) score_tile(std::integral_constant<int, h / 2>{}, std::false_type{});
                }
            }
            __syncthreads();
        }
    });

    // ---- final reference: the larger of the two groups' (and, in the variant that counts it, a positive
    // score beyond it); where a reference was raised on the way, numerators and accumulators follow ------
    if (tid < kFRow) {
        float m = fmaxf(Rtab[tid], Rtab[kFRow + tid]);
        if (bp.softmax_with_pos && tid < nrows && f_s[tid] - m > limit) {
            m = f_s[tid];
            flag_s[9] = 1u;
            if (!rescale_allowed) flag_s[8] = 1u;
        }
        ref_s[tid] = m;
    }
    __syncthreads();
    const bool raised = flag_s[9] != 0u;      // uniform
    // exp(reference of this wave's tile u - final reference) for rows 16r + 4g + v: 1 unless some
    // reference was raised on the way
    auto to_final = [&](int u, int r) __attribute__((always_inline)) {
        const float4 mf = lds4(ref_s + 16 * r + 4 * gq);
        const float4 rw = lds4(refw_of(grp, u, wl) + 16 * r + 4 * gq);
        return f32x4{fast_exp(rw.x - mf.x), fast_exp(rw.y - mf.y), fast_exp(rw.z - mf.z), fast_exp(rw.w - mf.w)};
    };

    // ---- row sums: over the sweep steps in registers, over 16 lanes, then over the waves --------
    {
        float* Lw = Ws;                       // [8 waves][64 rows]
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            f32x4 l = f32x4{0.f, 0.f, 0.f, 0.f};
            static_for<0, kFMaxSteps>([&](auto U) {
                constexpr int u = decltype(U)::value;
                if (tile_of(u) < ntiles) {
                    f32x4 t = P[u][r];
                    if (__builtin_expect(raised, 0)) t *= to_final(u, r);
                    l += t;
                }
            });
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float s = l[v];
                s += wave_shfl_xor(s, 1);
                s += wave_shfl_xor(s, 2);
                s += wave_shfl_xor(s, 4);
                s += wave_shfl_xor(s, 8);
                if (l15 == 0) Lw[w * kFRow + 16 * r + 4 * gq + v] = s;
            }
        }
    }
    __syncthreads();
    if (tid < kFRow) {
        const float* Lw = Ws;
        float sum = 0.f;
#pragma unroll
        for (int ww = 0; ww < kFWaves; ++ww) sum += Lw[ww * kFRow + tid];
        const bool live = tid < nrows;
        const float neg_sum = sum;
        if (bp.softmax_with_pos && live)      // Eq. 1 variant: the positive score is one more term of the sum
            sum += fast_exp_lifted(f_s[tid] - ref_s[tid]);
        // no reference exceeds its row's largest term, which therefore contributes at least 2^-58: the
        // sum can only leave this range if a score is not finite
        if (live && !(sum > 1e-30f && sum < 1e36f)) flag_s[8] = 1u;
        scale_s[tid] = live ? 1.f / sum : 0.f;
        logl_s[tid] = live ? logf(sum) : 0.f;
        // dL/df = minus the negatives' share of the sum (-1 as printed; no cancellation where the positive
        // dominates in the variant that counts it); the maxima kept here are no longer needed
        mx_s[tid] = live ? -neg_sum / sum : 0.f;
    }
    __syncthreads();
    const bool bad = flag_s[8] != 0u;
    if (tid == 0) {
        redo[blockIdx.x] = bad ? 1u : 0u;
        if (bad || raised) atomicAdd(redo_total, 1ull);
    }
    if (bad) return;                          // uniform: nothing has been written yet

    // ---- Q^T into LDS: QT[k][e]; the stored numerators become the softmax weights W = P / l ------
    float* QT = Ws;
    for (int idx = tid; idx < 16 * NJ * kFRow; idx += kFThreads) {
        const int e = idx & (kFRow - 1), k = idx >> 6;
        QT[k * kFQT + e] = k < d ? Qs[e * QS + k] : 0.f;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float4 sc4 = lds4(scale_s + 16 * r + 4 * gq);
        const f32x4 sc = f32x4{sc4.x, sc4.y, sc4.z, sc4.w};
        static_for<0, kFMaxSteps>([&](auto U) {
            constexpr int u = decltype(U)::value;
            if (tile_of(u) < ntiles) {
                f32x4 k = sc;
                if (__builtin_expect(raised, 0)) k *= to_final(u, r);
                P[u][r] *= k;
            }
        });
    }
    __syncthreads();

    // ---- G_neg, tile by tile; every wave works on its own 16 negatives, no workgroup barrier ------
    float* St = Ns + w * (16 * QS);           // private staging area, used as [16][d] without padding
    const float* qt = QT + l15 * kFQT + 4 * gq;
    static_for<0, kFMaxSteps>([&](auto U) {
        constexpr int u = decltype(U)::value;
        if (tile_of(u) < ntiles) {
            const int t = tile_of(u);
            f32x4 accC[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j) accC[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (16 * r < nrows) {
                    float4 b[NJ];
#pragma unroll
                    for (int j = 0; j < NJ; ++j) b[j] = lds4(qt + 16 * j * kFQT + 16 * r);
                    // step v contracts over rows 16r + 4g + v: nothing to add once 16r + v is past the chunk
#pragma unroll
                    for (int j = 0; j < NJ; ++j) accC[j] = mfma16(P[u][r][0], b[j].x, accC[j]);
                    if (16 * r + 1 < nrows) {
#pragma unroll
                        for (int j = 0; j < NJ; ++j) accC[j] = mfma16(P[u][r][1], b[j].y, accC[j]);
                    }
                    if (16 * r + 2 < nrows) {
#pragma unroll
                        for (int j = 0; j < NJ; ++j) accC[j] = mfma16(P[u][r][2], b[j].z, accC[j]);
                    }
                    if (16 * r + 3 < nrows) {
#pragma unroll
                        for (int j = 0; j < NJ; ++j) accC[j] = mfma16(P[u][r][3], b[j].w, accC[j]);
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int col = 16 * j + l15;
                if (col < d) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) St[(4 * gq + v) * d + col] = accC[j][v];
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // whole gradient rows leave as 16-byte pieces; row k of the staging area is negative
            // (16wl + k) * ntiles + t
#pragma unroll
            for (int s = 0; s < (16 * d / 4 + kWave - 1) / kWave; ++s) {
                const int idx = lane + kWave * s;
                const int k = idx / (d / 4);
                const int n = neg_of(t, 16 * wl + k);
                if (k < 16 && n < N)
                    *reinterpret_cast<float4*>(grad + (neg_base + n) * d + 4 * (idx - k * (d / 4))) = lds4(St + 4 * idx);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    });
    __syncthreads();

    // ---- epilogue: the two halves of G_Q to LDS, chain rule, gradient rows of the positives -----
    float* Gs = Ns + grp * (kFRow * QS);      // [2][64][QS]: one partial sum per wave group
    f32x4 down = f32x4{1.f, 1.f, 1.f, 1.f};   // this group's accumulators to the final reference
    if (__builtin_expect(raised, 0)) {
        const float4 ra = lds4(Rg + 16 * wl + 4 * gq), ma = lds4(ref_s + 16 * wl + 4 * gq);
        down = f32x4{fast_exp(ra.x - ma.x), fast_exp(ra.y - ma.y), fast_exp(ra.z - ma.z), fast_exp(ra.w - ma.w)};
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        float* grow = Gs + (16 * wl + 4 * gq + v) * QS;
#pragma unroll
        for (int q4 = 0; q4 < N4; ++q4)       // columns 64q + 4 l15 .. + 3 (all below d: d >= 64 N4)
            *reinterpret_cast<float4*>(grow + 64 * q4 + 4 * l15) =
                make_float4(accB[4 * q4][v] * down[v], accB[4 * q4 + 1][v] * down[v], accB[4 * q4 + 2][v] * down[v], accB[4 * q4 + 3][v] * down[v]);
        if constexpr (N2 == 1)
            *reinterpret_cast<float2*>(grow + 64 * N4 + 2 * l15) = make_float2(accB[4 * N4][v] * down[v], accB[4 * N4 + 1][v] * down[v]);
#pragma unroll
        for (int q1 = 0; q1 < N1; ++q1) {
            const int col = 64 * N4 + 32 * N2 + 16 * q1 + l15;
            if (col < d) grow[col] = accB[4 * N4 + 2 * N2 + q1][v] * down[v];
        }
    }
    __syncthreads();
    {
        int32_t ex[ITEMS], ey[ITEMS], er[ITEMS];
#pragma unroll
        for (int s = 0; s < ITEMS; ++s) {
            const bool live = it_row[s] < nrows;
            ex[s] = live ? eb[it_row[s] * 3 + xcol] : 0;
            ey[s] = live ? eb[it_row[s] * 3 + ycol] : 0;
            er[s] = live && SCORE != LEGEND_SCORE_DOT ? eb[it_row[s] * 3 + 1] : 0;
        }
        float x[ITEMS][4], y[ITEMS][4], r[ITEMS][4];
#pragma unroll
        for (int s = 0; s < ITEMS; ++s) {
            Item::load(Ex + (int64_t)ex[s] * d, it_c[s], x[s]);
            Item::load(Ey + (int64_t)ey[s] * d, it_c[s], y[s]);
            if (SCORE != LEGEND_SCORE_DOT) Item::load(bp.E_rel + (int64_t)er[s] * d, it_c[s], r[s]);
        }
#pragma unroll
        for (int s = 0; s < ITEMS; ++s) {
            if (it_row[s] < nrows) {
                const int row = it_row[s];
                const float sc = scale_s[row];
                const float a = mx_s[row];                // dL/df: -1 for Eq. 1 as printed
                float q[4], g0[4], g1[4], gv[4], gy4[4], gx4[4], gr4[4];
                Item::compose(side, x[s], r[s], q);
                Item::load(Ns + row * QS, it_c[s], g0);
                Item::load(Ns + (kFRow + row) * QS, it_c[s], g1);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    gv[t] = (g0[t] + g1[t]) * sc + a * y[s][t];
                    gy4[t] = a * q[t];
                }
                Item::chain(side, x[s], r[s], gv, gx4, gr4);
                const int64_t e = e0 + row;
                Item::store(grad + (side_base + (side == 0 ? 0 : g.P) + e) * d, it_c[s], gx4);
                Item::store(grad + (side_base + (side == 0 ? g.P : 0) + e) * d, it_c[s], gy4);
                if (SCORE != LEGEND_SCORE_DOT) Item::store(grad + (side_base + 2 * (int64_t)g.P + e) * d, it_c[s], gr4);
            }
        }
        if (tid < kFRow) rowloss_s[tid] = tid < nrows ? (ref_s[tid] - f_s[tid]) + (logl_s[tid] + kFLiftLn) : 0.f;   // lse - f
    }
    __syncthreads();
    if (tid == 0) {
        double s = 0.0;
        for (int r = 0; r < kFRow; ++r) s += (double)rowloss_s[r];
        loss_partial[blockIdx.x] = s;
    }
}

// Built for the dimension of the paper's large workloads and for d = 64 (the fully unrolled sweep is
// expensive to compile); every other shape takes the general kernel.  Each score function is
// compiled in a translation unit of its own (this file with LEGEND_FAST_SCORE set), so that the
// three compile side by side.
template <int SC, int D>
static hipError_t launch_fast_one(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    dim3 grid((unsigned)(g.sides * g.nchunks * g.T)), block(kFThreads);
    constexpr size_t lds = FastShape<D>::lds_bytes;
    static PerDeviceFlag configured;
    if (configured.pending()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_chunk_fast<SC, D>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured.set();
    }
    hipLaunchKernelGGL((k_chunk_fast<SC, D>), grid, block, lds, st, g, bp, ws.neg_ids, ws.grad,
                       ws.loss_partial, ws.redo, ws.redo_total, ws.fast_limit, ws.fast_no_rescale ? 0 : 1);
    return hipGetLastError();
}

template <int SC>
static hipError_t launch_fast_score(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    if (bp.dim == 100) return launch_fast_one<SC, 100>(st, g, bp, ws);
    if (bp.dim == 64) return launch_fast_one<SC, 64>(st, g, bp, ws);
    return hipErrorInvalidValue;
}

hipError_t launch_fast_dot(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws);
hipError_t launch_fast_distmult(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws);
hipError_t launch_fast_complex(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws);

#if LEGEND_FAST_SCORE == 0
hipError_t launch_fast_dot(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    return launch_fast_score<LEGEND_SCORE_DOT>(st, g, bp, ws);
}

bool chunk_fast_applies(const BatchGeom& g, const BucketParams& bp) {
    if (bp.loss != LEGEND_LOSS_SOFTMAX || bp.atomic_mode != 0) return false;
    if (g.N > 2 * kFMaxSteps * kFTile || g.N > kIdsLds || g.rows_tile > kFRow) return false;
    return bp.dim == 100 || bp.dim == 64;
}

hipError_t launch_chunks_fast(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    if (bp.score == LEGEND_SCORE_DOT) return launch_fast_dot(st, g, bp, ws);
    if (bp.score == LEGEND_SCORE_DISTMULT) return launch_fast_distmult(st, g, bp, ws);
    return launch_fast_complex(st, g, bp, ws);
}
#elif LEGEND_FAST_SCORE == 1
hipError_t launch_fast_distmult(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    return launch_fast_score<LEGEND_SCORE_DISTMULT>(st, g, bp, ws);
}
#else
hipError_t launch_fast_complex(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    return launch_fast_score<LEGEND_SCORE_COMPLEX>(st, g, bp, ws);
}
#endif

}  // namespace legend
