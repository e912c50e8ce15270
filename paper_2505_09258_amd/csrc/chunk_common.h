// Device helpers shared by the chunk kernels (narrow: dim <= 128, wide: dim <= 512).
#pragma once

#include <hip/hip_runtime.h>

#include "legend_internal.h"
#include "device_utils.h"

namespace legend {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kChunkThreads = 256;
constexpr int kIdsLds = 1024;   // negative ids of a chunk kept in LDS (more than that: read from global)
constexpr int kNarrowMaxDim = 128;
constexpr int kWideMaxDim = 512;
constexpr int kWideRowTile = 112;  // rows of positives per tile for dim > 128 (seven 16-row MFMA blocks)

// LDS row stride of the Q and negative tiles: dim rounded up to 8, plus 4.  It is a multiple
// of 4 (rows stay 16-byte aligned for 128-bit LDS accesses) and 4 mod 8 (32 rows read at the
// same column fall into distinct bank groups).
__host__ __device__ inline int chunk_row_stride(int d) { return ((d + 7) & ~7) + 4; }

__device__ inline f32x16 mfma32(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ inline float softplusf(float x) {
    // log(1 + exp(x)) without overflow
    return fmaxf(x, 0.f) + log1pf(expf(-fabsf(x)));
}
__device__ inline float sigmoidf(float x) { return 1.f / (1.f + expf(-x)); }

// exp(x) for finite x from the hardware 2^x instruction: the product x * log2(e) is formed in
// two pieces (head, and rounding error + low part of the constant) so that the result is good
// to about two ulp for any magnitude of x, at six VALU instructions.
__device__ inline float fast_exp(float x) {
    const float L2E_HI = 1.44269502162933349609375f;
    const float L2E_LO = 1.925963033500011e-8f;
    const float hi = x * L2E_HI;
    float lo = fmaf(x, L2E_HI, -hi);
    lo = fmaf(x, L2E_LO, lo);
    const float r = __builtin_amdgcn_exp2f(hi);
    return fmaf(r, lo * 0.6931471805599453f, r);
}

__device__ inline float4 lds4(const float* p) { return *reinterpret_cast<const float4*>(p); }

// MFMA operand mapping used by the chunk kernels: the contraction index runs in groups of 8;
// in a group the lanes 0-31 (kk = 0) supply k = 8g + s and lanes 32-63 (kk = 1) supply
// k = 8g + 4 + s to the s-th of four consecutive 32x32x2 MFMAs (s = 0..3).  Both operands
// use the same mapping, so the sum over k is complete and every lane can fetch its four
// values of a row-major operand with one 128-bit LDS read.

bool chunk_fast_applies(const BatchGeom& g, const BucketParams& bp);
hipError_t launch_chunks_fast(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws);
hipError_t launch_chunks_trans(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws);
hipError_t launch_chunks_gemm(hipStream_t st, const BatchGeom& g, const BucketParams& bp, const Workspace& ws);

}  // namespace legend
