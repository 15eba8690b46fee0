// Building blocks for dense layers on the gfx950 matrix cores (fp32 path).
//
// v_mfma_f32_32x32x2_f32: one wavefront multiplies A[32][2] by B[2][32] and
// accumulates into D[32][32].  Lane l supplies A[l%32][l/32] and
// B[l/32][l%32]; it owns D[8*(i/4) + 4*(l/32) + i%4][l%32] for i = 0..15.
//
// Activations ("A tile") live in LDS as planes of 16-byte entries: plane q holds
// columns 4q..4q+3 (fp32) or 8q..8q+7 (bf16) of every row, plane stride = rows + 1
// entries (the +1 keeps consecutive planes on different banks).  Weights come straight from global
// memory in the PackedLayer order, where one float4 per lane per k-group is a
// fully coalesced 1 KiB read per wavefront.
#pragma once
#include <hip/hip_runtime.h>

namespace dkf {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f32x16 mfma32(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

// row (0..31) of accumulator element i held by `lane`
__device__ __forceinline__ int acc_row(int i, int lane) { return (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3); }

// ---- A tiles in LDS --------------------------------------------------------------
// fp32: planes of 4 columns (one float4 per row); bf16: planes of 8 columns (eight bf16 =
// 16 bytes per row).  Either way a plane entry is 16 bytes and the plane stride is `lda`
// entries, so both element types share buffers and index arithmetic.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <bool BF16>
__device__ __forceinline__ void tile_put(f32x4 *tile, int lda, int row, int col, float v) {
    if constexpr (BF16)
        reinterpret_cast<__bf16 *>(tile)[((col >> 3) * lda + row) * 8 + (col & 7)] = (__bf16)v;  // round to nearest even
    else
        reinterpret_cast<float *>(tile)[((col >> 2) * lda + row) * 4 + (col & 3)] = v;
}

__device__ __forceinline__ f32x16 mfma32_bf16(f32x4 a, f32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0,
                                                   0);
}

// acc += A[rows r0..r0+31][k-groups kg0..kg1) * layer column block `tiles_nb`.
// tiles_nb points at the [k_groups][64] 16-byte entries of one 32-column block.  A k-group
// is 8 columns in fp32 (four v_mfma_f32_32x32x2_f32) and 16 columns in bf16 (one
// v_mfma_f32_32x32x16_bf16: lane l supplies row/column l%32 and k = 8*(l/32)..+7).
template <bool BF16>
__device__ __forceinline__ void mma_block(f32x16 &acc, const f32x4 *A, int lda, int r0,
                                          const f32x4 *__restrict__ tiles_nb, int kg0, int kg1, int lane) {
    const int r = r0 + (lane & 31), half = lane >> 5;
#pragma unroll 4
    for (int kg = kg0; kg < kg1; ++kg) {
        const f32x4 b = tiles_nb[kg * 64 + lane];
        const f32x4 a = A[(kg * 2 + half) * lda + r];
        if constexpr (BF16) {
            acc = mfma32_bf16(a, b, acc);
        } else {
            acc = mfma32(a.x, b.x, acc);
            acc = mfma32(a.y, b.y, acc);
            acc = mfma32(a.z, b.z, acc);
            acc = mfma32(a.w, b.w, acc);
        }
    }
}

// Nonlinearities on the hardware exp2 / log2 / reciprocal units (about 1 ulp each; the absolute
// error of every function below stays under 3e-7 of its range).  The raw instructions are used:
// exp2 of a large negative argument flushes to zero, which is the right limit here, and the
// logarithm's argument lies in [1, 2], so neither needs the library's denormal handling.
__device__ __forceinline__ float fast_rcp(float v) { return __builtin_amdgcn_rcpf(v); }
__device__ __forceinline__ float exp_f(float v) { return __builtin_amdgcn_exp2f(v * 1.44269504088896341f); }
__device__ __forceinline__ float tanh_f(float v) {  // 1 - 2 / (exp(2v) + 1)
    return 1.0f - 2.0f * fast_rcp(__builtin_amdgcn_exp2f(v * 2.88539008177792681f) + 1.0f);
}
__device__ __forceinline__ float softplus_f(float v) {  // max(v, 0) + ln(1 + exp(-|v|))
    const float e = __builtin_amdgcn_exp2f(fabsf(v) * -1.44269504088896341f);
    // (max(v, 0) as a median of three: fmaxf costs a second instruction that quiets signalling NaNs)
    return __builtin_amdgcn_fmed3f(v, 0.f, __builtin_huge_valf()) + 0.693147180559945309f * __builtin_amdgcn_logf(1.0f + e);
}
__device__ __forceinline__ float sigmoid_f(float v) {
    const float e = __builtin_amdgcn_exp2f(fabsf(v) * -1.44269504088896341f);
    const float r = fast_rcp(1.0f + e);
    return v >= 0.f ? r : e * r;
}

}  // namespace dkf
