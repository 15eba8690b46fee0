// Sorting network for one row of run-times held in the registers of a lane group (Sec. 3.1.1, last
// paragraph: the Monte-Carlo estimate of the order statistics sorts every sampled vector).  Shared by
// the row-sort kernel and by the sampler that sorts its own rows before they leave the compute unit.
// Keys are the order-preserving uint32 image of the fp32 bits, so all compares are integer min/max.
#pragma once
#include "common.h"

namespace dkf {
namespace {

constexpr uint32_t kPadKey = 0xFFFFFFFFu;
constexpr uint32_t kNanKey = 0xFFFFFFFEu;

__device__ __forceinline__ uint32_t key_of(float x) {
    uint32_t u = __float_as_uint(x);
    if (x != x) return kNanKey;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float value_of(uint32_t k) {
    uint32_t u = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    return __uint_as_float(u);
}

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v / 2); }

// A row is held by a lane group of G = 2^LG lanes with E keys each.  Position p = e + E * g of
// the sorting network belongs to key register e of lane g: the low log2(E) bits of a position are
// register bits, so the network's stages on those bits -- the ones that occur most often -- are
// compare-exchanges between registers of one lane, and only the stages on the high bits cross
// lanes.  Where a key sits when it is loaded does not matter to a sort, so the row is read with
// whichever pattern coalesces best (load_index: one float4 per lane and instruction, consecutive
// lanes on consecutive 16 bytes); after the network position p holds rank p.
template <int E, int LG>
struct Layout {
    static constexpr int kLgE = ilog2(E);
    static constexpr int kLgN = kLgE + LG;
    __host__ __device__ static constexpr bool is_lane_bit(int b) { return b >= kLgE; }
    __host__ __device__ static constexpr int reg_bit(int b) { return b; }
    __host__ __device__ static constexpr int lane_bit(int b) { return b - kLgE; }
    // masks of the low m position bits, split into key-register and lane parts
    __host__ __device__ static constexpr int reg_mask(int m) {
        int r = 0;
        for (int b = 0; b < m; ++b)
            if (!is_lane_bit(b)) r |= 1 << reg_bit(b);
        return r;
    }
    __host__ __device__ static constexpr int lane_mask(int m) {
        int r = 0;
        for (int b = 0; b < m; ++b)
            if (is_lane_bit(b)) r |= 1 << lane_bit(b);
        return r;
    }
    // index in the row of the key that register e of lane g loads
    __device__ static __forceinline__ int load_index(int g, int e) {
        return (e & 3) | (g << 2) | ((e >> 2) << (2 + LG));
    }
    // rank held by register e of lane g after the network
    __device__ static __forceinline__ int rank(int g, int e) { return e | (g << kLgE); }
};

template <typename T>
__device__ __forceinline__ T tmin(T a, T b) { return a < b ? a : b; }
template <typename T>
__device__ __forceinline__ T tmax(T a, T b) { return a < b ? b : a; }

// ---- cross-lane exchanges of 32-bit keys without the LDS crossbar where possible ---------
// DPP moves reach lane ^ 1, ^ 2, ^ 8 and the mirror images inside 4, 8 and 16 lanes directly and
// lane ^ 4 as two mirrors; only distances 16 and 32 go through ds_bpermute.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
// value of lane ^ LM for LM = 2^k, or of lane ^ LM for LM = 2^k - 1 (mirror inside 2^k lanes)
template <int LM>
__device__ __forceinline__ uint32_t from_lane_xor(uint32_t x) {
    if constexpr (LM == 1) return dpp_mov<0xB1>(x);                      // quad_perm [1,0,3,2]
    else if constexpr (LM == 2) return dpp_mov<0x4E>(x);                 // quad_perm [2,3,0,1]
    else if constexpr (LM == 3) return dpp_mov<0x1B>(x);                 // quad_perm [3,2,1,0]
    else if constexpr (LM == 4) return dpp_mov<0x1B>(dpp_mov<0x141>(x)); // (l ^ 7) ^ 3
    else if constexpr (LM == 7) return dpp_mov<0x141>(x);                // row_half_mirror
    else if constexpr (LM == 8) return dpp_mov<0x128>(x);                // row_ror:8
    else if constexpr (LM == 15) return dpp_mov<0x140>(x);               // row_mirror
    else return (uint32_t)__shfl_xor((int)x, LM, 64);
}
// median of three: with c = 0 it is min(a, b), with c = 0xFFFFFFFF it is max(a, b), so one
// instruction serves the lanes that keep the smaller key and those that keep the larger one
// (written as the min/max form the compiler selects v_med3_u32 for: after an asm block it would
// pad every following DPP move with wait states it cannot prove unnecessary)
__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c) {
    const uint32_t lo = a < b ? a : b, hi = a < b ? b : a;
    const uint32_t t = lo < c ? c : lo;  // max(min(a, b), c)
    return t < hi ? t : hi;              // min(., max(a, b))
}
// Compare-exchange with lane ^ 4 for K keys, two instructions per key.  No single DPP pattern is
// lane ^ 4, but a rotation by four inside the row of 16 lanes reaches it from one side: lanes whose
// bit 2 is clear find their partner four lanes up (row_ror:12), the others four lanes down
// (row_ror:4).  v_min_u32 / v_max_u32 take the DPP operand directly, and the bank mask lets each of
// them write only the lanes it is right for (banks 0 and 2 keep the minimum, 1 and 3 the maximum).
// The leading s_nop covers the two wait states a DPP read needs after a vector write of the same
// register, which the compiler cannot see inside an asm block.
#define DKF_X4(i) "v_min_u32_dpp %" #i ", %[x" #i "], %[x" #i "] row_ror:12 row_mask:0xf bank_mask:0x5\n\t" \
                  "v_max_u32_dpp %" #i ", %[x" #i "], %[x" #i "] row_ror:4 row_mask:0xf bank_mask:0xa\n\t"
__device__ __forceinline__ void exchange_xor4(uint32_t (&v)[4]) {
    uint32_t r0, r1, r2, r3;
    asm volatile("s_nop 1\n\t" DKF_X4(0) DKF_X4(1) DKF_X4(2) DKF_X4(3)
                 : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3)
                 : [x0] "v"(v[0]), [x1] "v"(v[1]), [x2] "v"(v[2]), [x3] "v"(v[3]));
    v[0] = r0; v[1] = r1; v[2] = r2; v[3] = r3;
}
#undef DKF_X4
// 0 in lanes whose group-lane bit `bit` is clear (they keep the minimum), all ones in the others
__device__ __forceinline__ uint32_t keep_mask(int g, int bit) { return (g >> bit) & 1 ? 0xFFFFFFFFu : 0u; }

// Compare-exchange across element bit B (partner = i ^ 2^B); the element whose
// bit B is clear keeps the smaller key.
template <typename T, int E, int LG, int B>
__device__ __forceinline__ void xor_stage(T (&v)[E], int g) {
    using Lay = Layout<E, LG>;
    if constexpr (Lay::is_lane_bit(B)) {
        constexpr int lm = 1 << Lay::lane_bit(B);
        if constexpr (sizeof(T) == 4 && lm == 4 && E % 4 == 0) {
#pragma unroll
            for (int e = 0; e < E; e += 4) {
                uint32_t q[4] = {v[e], v[e + 1], v[e + 2], v[e + 3]};
                exchange_xor4(q);
                v[e] = q[0]; v[e + 1] = q[1]; v[e + 2] = q[2]; v[e + 3] = q[3];
            }
        } else if constexpr (sizeof(T) == 4) {
            const uint32_t sel = keep_mask(g, Lay::lane_bit(B));
            // all moves first, then all medians: a DPP move that reads a register the instruction
            // just before it wrote costs wait states
            uint32_t p[E];
#pragma unroll
            for (int e = 0; e < E; ++e) p[e] = from_lane_xor<lm>(v[e]);
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = umed3(v[e], p[e], sel);
        } else {
            const bool keep_min = (g & lm) == 0;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                T p = __shfl_xor(v[e], lm, 64);
                v[e] = keep_min ? tmin(v[e], p) : tmax(v[e], p);
            }
        }
    } else {
        constexpr int rm = 1 << Lay::reg_bit(B);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if ((e & rm) == 0) {
                T a = v[e], b = v[e | rm];
                v[e] = tmin(a, b);
                v[e | rm] = tmax(a, b);
            }
        }
    }
}

// First stage of merging two sorted runs of 2^(M-1): partner = i ^ (2^M - 1).
template <typename T, int E, int LG, int M>
__device__ __forceinline__ void flip_stage(T (&v)[E], int g) {
    using Lay = Layout<E, LG>;
    constexpr int rm = Lay::reg_mask(M);
    constexpr int lm = Lay::lane_mask(M);
    constexpr int top = M - 1;
    if constexpr (lm == 0) {
        constexpr int tb = 1 << Lay::reg_bit(top);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if ((e & tb) == 0) {
                T a = v[e], b = v[e ^ rm];
                v[e] = tmin(a, b);
                v[e ^ rm] = tmax(a, b);
            }
        }
    } else {
        T p[E];
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int e = 0; e < E; ++e) p[e] = from_lane_xor<lm>(v[e ^ rm]);
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) p[e] = __shfl_xor(v[e ^ rm], lm, 64);
        }
        if constexpr (Lay::is_lane_bit(top)) {
            if constexpr (sizeof(T) == 4) {
                const uint32_t sel = keep_mask(g, Lay::lane_bit(top));
#pragma unroll
                for (int e = 0; e < E; ++e) v[e] = umed3(v[e], p[e], sel);
            } else {
                const bool keep_min = (g & (1 << Lay::lane_bit(top))) == 0;
#pragma unroll
                for (int e = 0; e < E; ++e) v[e] = keep_min ? tmin(v[e], p[e]) : tmax(v[e], p[e]);
            }
        } else {
            constexpr int tb = 1 << Lay::reg_bit(top);
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = (e & tb) == 0 ? tmin(v[e], p[e]) : tmax(v[e], p[e]);
        }
    }
}

template <typename T, int E, int LG, int B>
__device__ __forceinline__ void xor_down(T (&v)[E], int g) {
    if constexpr (B >= 0) {
        xor_stage<T, E, LG, B>(v, g);
        xor_down<T, E, LG, B - 1>(v, g);
    }
}

// The keys of one lane sorted by Batcher's odd-even merge sort (ascending in register order):
// between registers any pairing costs the same, and this network needs a fifth fewer
// compare-exchanges than the bitonic one (19 against 24 for 8 keys, 191 against 240 for 32).
template <typename T, int E>
__device__ __forceinline__ void sort_in_lane(T (&v)[E]) {
#pragma unroll
    for (int p = 1; p < E; p *= 2) {
#pragma unroll
        for (int k = p; k >= 1; k /= 2) {
#pragma unroll
            for (int j = k % p; j + k < E; j += 2 * k) {
#pragma unroll
                for (int i = 0; i < k; ++i) {
                    const int lo = i + j, hi = i + j + k;
                    if (hi < E && lo / (2 * p) == hi / (2 * p)) {
                        const T a = v[lo], b = v[hi];
                        v[lo] = tmin(a, b);
                        v[hi] = tmax(a, b);
                    }
                }
            }
        }
    }
}

template <typename T, int E, int LG, int M>
__device__ __forceinline__ void merge_up(T (&v)[E], int g) {
    if constexpr (M <= Layout<E, LG>::kLgN) {
        flip_stage<T, E, LG, M>(v, g);
        xor_down<T, E, LG, M - 2>(v, g);
        merge_up<T, E, LG, M + 1>(v, g);
    }
}

// key_of as straight-line code: exclusive-or with the sign spread over the word and the top bit
__device__ __forceinline__ uint32_t key_of_flat(float x) {
    const uint32_t u = __float_as_uint(x);
    const uint32_t k = u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
    return x != x ? kNanKey : k;
}

}  // namespace
}  // namespace dkf
