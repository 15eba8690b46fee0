// Built-in standard-normal noise for the three reparameterised draws of the sampler
// (guide steps, transition, emission; Sec. 3.1.3), used when the caller supplies no tensors.
//
// Counter-based: element i of tensor t (0 = eps_q, 1 = eps_z, 2 = eps_x) is the (i mod 4)-th
// output of Box-Muller applied to Philox4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel random
// numbers: as easy as 1, 2, 3", SC'11) with counter (i/4 low, i/4 high, t, 0) and key
// (seed low, seed high).  Uniforms use the top 24 bits of each word, u1 = (w0 >> 8) + 1) / 2^24
// in (0, 1], u2 = (w1 >> 8) / 2^24 in [0, 1), so both are exact in fp32:
//   n0 = sqrt(-2 ln u1) cos(2 pi u2), n1 = sqrt(-2 ln u1) sin(2 pi u2); words 2, 3 give n2, n3.
#include "common.h"

namespace dkf {
namespace {

struct U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // (each 64-bit product written as one: a single multiply instruction yields both halves)
        const uint64_t p0 = (uint64_t)0xD2511F53u * c.x, p1 = (uint64_t)0xCD9E8D57u * c.z;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        c = U4{hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0};
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c;
}

__device__ __forceinline__ void box_muller(uint32_t w0, uint32_t w1, float &n0, float &n1) {
    const float u1 = (float)((w0 >> 8) + 1u) * (1.0f / 16777216.0f);
    const float u2 = (float)(w1 >> 8) * (1.0f / 16777216.0f);
    // hardware log2 / sqrt / sin / cos (the last two take their argument in revolutions, which is
    // what u2 is): u1 is a normal number in (0, 1] and u2 lies in [0, 1), so none of the library
    // routines' range handling is needed; absolute error of a normal about 1e-6
    const float r = __builtin_amdgcn_sqrtf(-1.38629436111989062f * __builtin_amdgcn_logf(u1));  // -2 ln u1 = -2 ln 2 log2 u1
    n0 = r * __builtin_amdgcn_cosf(u2);
    n1 = r * __builtin_amdgcn_sinf(u2);
}

// four consecutive elements 4g .. 4g+3 of tensor `tensor`
__device__ __forceinline__ void fill_group(float *__restrict__ out, size_t n, uint32_t tensor, size_t g,
                                           uint32_t seed_lo, uint32_t seed_hi) {
    const U4 r = philox4x32_10(U4{(uint32_t)g, (uint32_t)(g >> 32), tensor, 0u}, seed_lo, seed_hi);
    float v[4];
    box_muller(r.x, r.y, v[0], v[1]);
    box_muller(r.z, r.w, v[2], v[3]);
    const size_t i0 = g * 4;
    if (i0 + 3 < n) {
        *reinterpret_cast<float4 *>(out + i0) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        for (int j = 0; j < 4; ++j)
            if (i0 + j < n) out[i0 + j] = v[j];
    }
}

// Tensors 0, 1, 2 in one launch, one thread per group of four elements; the groups of the three
// tensors are numbered one after the other.
__global__ __launch_bounds__(256) void fill_normal3(float *__restrict__ out0, size_t n0, float *__restrict__ out1,
                                                    size_t n1, float *__restrict__ out2, size_t n2,
                                                    const Control *ctl, uint32_t seed_lo, uint32_t seed_hi) {
    if (ctl) { seed_lo = ctl->seed_lo; seed_hi = ctl->seed_hi; }
    const size_t g0 = (n0 + 3) / 4, g1 = (n1 + 3) / 4, g2 = (n2 + 3) / 4;
    for (size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x; g < g0 + g1 + g2; g += (size_t)gridDim.x * blockDim.x) {
        if (g < g0) fill_group(out0, n0, 0u, g, seed_lo, seed_hi);
        else if (g < g0 + g1) fill_group(out1, n1, 1u, g - g0, seed_lo, seed_hi);
        else fill_group(out2, n2, 2u, g - g0 - g1, seed_lo, seed_hi);
    }
}

}  // namespace

int launch_fill_normal3(float *out0, size_t n0, float *out1, size_t n1, float *out2, size_t n2, const Control *ctl,
                        uint64_t seed, hipStream_t stream) {
    if (!out0 || !out1 || !out2) return DKF_EINVAL;
    const size_t groups = (n0 + 3) / 4 + (n1 + 3) / 4 + (n2 + 3) / 4;
    if (groups == 0) return DKF_OK;
    size_t blocks = (groups + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_normal3, dim3((unsigned)blocks), dim3(256), 0, stream, out0, n0, out1, n1, out2, n2, ctl,
                       (uint32_t)seed, (uint32_t)(seed >> 32));
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

}  // namespace dkf
