// Building blocks shared by the kernels that chain layers through v_mfma_f32_16x16x4_f32 with the
// weights as the A operand (16 output features x 4 input features per instruction) and the
// activations as the B operand (4 input features x 16 samples): lane l of an activation block
// holds features 4 (l / 16) + v, v = 0..3, of sample l % 16, which is both what a result block
// looks like and what the next layer's instructions consume (instruction v takes register v).
// A weight tile is 64 lanes x float4: lane 16 q + i holds W[16 ob + i][16 ib + 4 q .. + 3].
#pragma once
#include "mfma_tile.h"

namespace dkf {
namespace {

__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Keeps the instruction scheduler from hoisting later blocks' operand loads above this point
// (otherwise dozens of weight tiles are prefetched into registers and the kernel spills).
__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

__device__ __forceinline__ f32x4 splat(float v) { f32x4 r = {v, v, v, v}; return r; }

template <typename F>
__device__ __forceinline__ f32x4 map4(f32x4 v, F f) {
    f32x4 r = {f(v.x), f(v.y), f(v.z), f(v.w)};
    return r;
}

// Calls use(g, tiles) for every group of GROUP consecutive tiles (COUNT must be a multiple of
// GROUP).  The next group is already being fetched while the current one feeds the matrix
// cores; the scheduling fence after each group bounds how far ahead the compiler may hoist
// operand loads (unbounded hoisting spills).
template <int COUNT, int GROUP, typename LoadF, typename UseG>
__device__ __forceinline__ void for_tile_groups(LoadF &&load, UseG &&use) {
    static_assert(COUNT % GROUP == 0, "whole groups");
    constexpr int kGroups = COUNT / GROUP;
    f32x4 buf[2][GROUP];
#pragma unroll
    for (int j = 0; j < GROUP; ++j) buf[0][j] = load(j);
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
        if (g + 1 < kGroups) {
#pragma unroll
            for (int j = 0; j < GROUP; ++j) buf[(g + 1) & 1][j] = load((g + 1) * GROUP + j);
        }
        use(g, buf[g & 1]);
        sched_fence();
    }
}

// A dependent v_mfma_f32_16x16x4_f32 cannot issue until its predecessor has left the pipe, so
// every product below is spread over four accumulator chains that advance in turn.

// GROUP output blocks, one tile each, same input block x:  out[j] += W_j x
template <int GROUP>
__device__ __forceinline__ void mma_wide(f32x4 *out, const f32x4 (&t)[GROUP], f32x4 x) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int j = 0; j < GROUP; ++j) out[j] = mfma16(t[j][e], x[e], out[j]);
}

// one output block accumulated over GROUP input blocks in C chains (k-slice e of a tile goes to
// chain e % C); the chains are added in a fixed order at the end
template <int C>
struct Acc {
    static_assert(C == 1 || C == 2 || C == 4, "chains");
    f32x4 c[C];
    __device__ __forceinline__ void init(f32x4 first) {
        c[0] = first;
#pragma unroll
        for (int i = 1; i < C; ++i) c[i] = splat(0.f);
    }
    __device__ __forceinline__ f32x4 sum() const {
        if constexpr (C == 4) return (c[0] + c[1]) + (c[2] + c[3]);
        else if constexpr (C == 2) return c[0] + c[1];
        else return c[0];
    }
};
using Acc4 = Acc<4>;
template <int GROUP, int C>
__device__ __forceinline__ void mma_narrow(Acc<C> &acc, const f32x4 (&t)[GROUP], const f32x4 *x) {
#pragma unroll
    for (int j = 0; j < GROUP; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc.c[e % C] = mfma16(t[j][e], x[j][e], acc.c[e % C]);
}

}  // namespace
}  // namespace dkf
