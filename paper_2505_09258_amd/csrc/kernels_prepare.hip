// Batch construction on the GPU (paper Sec. 2.1 stages 1-2, Sec. 3 step 3):
// negative ids from a counter hash and the sort key of every gradient row.
#include "legend_internal.h"
#include "device_utils.h"

namespace legend {

__global__ void __launch_bounds__(256)
k_validate_edges(const int32_t* __restrict__ edges, int64_t m, int32_t rows_src, int32_t rows_dst,
                 int32_t num_rel, int check_rel, uint32_t* __restrict__ err_flag) {
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (; e < m; e += stride) {
        int32_t s = edges[e * 3 + 0], r = edges[e * 3 + 1], d = edges[e * 3 + 2];
        bad |= (s < 0) | (s >= rows_src) | (d < 0) | (d >= rows_dst);
        if (check_rel) bad |= (r < 0) | (r >= num_rel);
    }
    if (bad) atomicOr(err_flag, 1u);
}

hipError_t launch_validate_edges(hipStream_t st, const int32_t* edges, int64_t m, int32_t rows_src,
                                 int32_t rows_dst, int32_t num_rel, int check_rel, uint32_t* err_flag) {
    if (m <= 0) return hipSuccess;
    int64_t blocks = (m + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_validate_edges, dim3((unsigned)blocks), dim3(256), 0, st, edges, m, rows_src, rows_dst,
                       num_rel, check_rel, err_flag);
    return hipGetLastError();
}

// Plain fill of 32-bit words: clears counters and flags where a memset node must not be recorded.
__global__ void __launch_bounds__(256) k_fill_u32(uint32_t* __restrict__ p, uint32_t v, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

hipError_t launch_fill_u32(hipStream_t st, uint32_t* p, uint32_t v, int64_t n) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, st, p, v, n);
    return hipGetLastError();
}

// Seeded initial embeddings ("randomly initialized", Sec. 3 step 1; the distribution is not printed):
// element (row g, column k) of a table is a pure integer function of (seed, table tag, g, k),
//     h = fold(fold(fold(seed, tag), g), k),   u = sum of the four 16-bit fields of h  (0 .. 262140),
//     value = float(int(u) - 131070) * scale,  scale = float(init_std * sqrt(3) / 65536),
// a sum of four uniform integers: mean 0, standard deviation init_std, no transcendental function.
__global__ void __launch_bounds__(256)
k_init_fill(float* __restrict__ out, int64_t rows, int32_t dim, int64_t row0, uint64_t table_hash, float scale) {
    const int64_t total = rows * dim;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const int64_t r = idx / dim;
        const int k = (int)(idx - r * dim);
        const uint64_t h = hash_fold(hash_fold(table_hash, (uint64_t)(row0 + r)), (uint64_t)k);
        const int32_t u = (int32_t)((h & 0xFFFFu) + ((h >> 16) & 0xFFFFu) + ((h >> 32) & 0xFFFFu) + (h >> 48));
        out[idx] = (float)(u - 131070) * scale;
    }
}

hipError_t launch_init_fill(hipStream_t st, float* out, int64_t rows, int32_t dim, int64_t row0, uint64_t seed,
                            uint64_t table_tag, float init_std) {
    if (rows <= 0) return hipSuccess;
    const float scale = (float)((double)init_std * 1.7320508075688772 / 65536.0);
    int64_t blocks = (rows * dim + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(k_init_fill, dim3((unsigned)blocks), dim3(256), 0, st, out, rows, dim, row0,
                       hash_fold(seed, table_tag), scale);
    return hipGetLastError();
}

// One thread per occurrence (gradient row) of the batch: its sort key, and for
// negative rows the sampled id.  Index arithmetic only; no floating point.
__global__ void __launch_bounds__(256)
k_prepare(BatchGeom g, BucketParams bp, int32_t* __restrict__ neg_ids, uint32_t* __restrict__ keys) {
    int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= g.n_occ) return;
    int si = (int)(o / g.per_side);
    int64_t r = o - (int64_t)si * g.per_side;
    int side = g.side_id[si];
    const int32_t* eb = bp.edges + bp.batch_lo * 3;
    uint32_t key;
    if (r < g.P) {
        key = (uint32_t)eb[r * 3 + 0];
    } else if (r < 2 * (int64_t)g.P) {
        key = bp.key_base_dst + (uint32_t)eb[(r - g.P) * 3 + 2];
    } else if (g.roles == 3 && r < 3 * (int64_t)g.P) {
        key = bp.key_base_rel + (uint32_t)eb[(r - 2 * (int64_t)g.P) * 3 + 1];
    } else {
        int64_t q = r - (int64_t)g.roles * g.P;
        int k = (int)(q % g.N);
        int64_t ct = q / g.N;
        int t = (int)(ct % g.T);
        int c = (int)(ct / g.T);
        uint64_t h = hash_fold(hash_fold(hash_fold(bp.hash_prefix, (uint64_t)c), (uint64_t)side), (uint64_t)k);
        int32_t id;
        if (k < g.N - bp.num_degree_negs) {
            uint64_t rows = (uint64_t)(side == 0 ? bp.rows_valid_dst : bp.rows_valid_src);
            id = (int32_t)__umul64hi(h, rows);
        } else {
            uint64_t e = __umul64hi(h, (uint64_t)bp.m);
            id = bp.edges[e * 3 + (side == 0 ? 2 : 0)];
        }
        key = (side == 0 ? bp.key_base_dst : 0u) + (uint32_t)id;
        if (t == 0) neg_ids[((int64_t)si * g.nchunks + c) * g.N + k] = id;
    }
    keys[o] = key;
}

hipError_t launch_prepare(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws) {
    if (g.n_occ <= 0) return hipSuccess;
    unsigned blocks = (unsigned)((g.n_occ + 255) / 256);
    hipLaunchKernelGGL(k_prepare, dim3(blocks), dim3(256), 0, st, g, bp, ws.neg_ids, ws.keys[0]);
    return hipGetLastError();
}

}  // namespace legend
