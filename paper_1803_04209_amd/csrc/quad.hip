// Posterior-predictive sampling for small sample counts (Sec. 3.1.3): the same chain of layers
// as chain.hip -- L guide steps, the gated transition draw, the emission draw -- but with FOUR
// samples per wavefront instead of sixteen, so that a few thousand samples still put one
// wavefront on every SIMD of the chip.  (With sixteen samples per wavefront, 4096 samples are
// 256 wavefronts: one per SIMD on a quarter of the compute units, each bound by its own chain
// of dependent layers.)
//
// Matrix instruction: v_mfma_f32_4x4x1_16b_f32, sixteen independent 4x4 outer products per issue.
// Lane 4b+i of the A operand is row i of block b, lane 4b+j of the B operand is column j of
// block b, and register i, lane 4b+j of the result is D_b[i][j].  Rows are the four samples,
// columns are output features, and the broadcast field of the instruction lets one block of
// A serve several blocks of B:
//   wide layer   (64 outputs per instruction): A block `abid` is broadcast to all 16 blocks;
//                B lane l carries W[64 og + l][k].  One instruction = 4 samples x 64 outputs
//                x one input feature k.
//   narrow layer (16 outputs per instruction): blocks are 4 groups of 4; group g takes A block
//                4g + abid, i.e. a different input feature per group, so the instruction covers
//                four input features at once and leaves four partial sums per output (one per
//                group of 16 lanes) that two lane-swap instructions and three adds combine.
//
// Register layouts of an activation (4 samples x features):
//   D (result of a wide layer, per 64-feature group): register i = sample i, lane l = feature l
//   A (input of a layer, per 64-feature group):       register j, lane 4b+i = feature 4b+j of
//                                                     sample i  (a 4x4 transpose of D inside
//                                                     every quad of lanes: four DPP moves + selects)
//   P (result of a narrow layer, per 16 features):    one register, lane 16r+k = feature k of
//                                                     sample sigma(r), sigma = (0, 2, 1, 3)
//   Q (narrow input, per 16 features):                one register, lane 4k+i = feature k of sample i
//                                                     (from P by one lane permutation)
// Weight tiles (64 lanes x float4 = 1 KiB = four instructions' B operands) are laid out for
// exactly these pairings when the weights are loaded (pack_quad, api.hip).
//
// Guide weights stay in LDS for the L steps; the transition and emission weights are streamed
// once per workgroup (four wavefronts = 16 samples) from L2 through a ring of LDS buffers.
#include <type_traits>

#include "common.h"
#include "mfma_tile.h"

namespace dkf {
namespace {

constexpr int kThreads = 256;
constexpr int kTileF4 = 64;
constexpr int CH = kQuadChunkTiles;
constexpr int kChunkF4 = CH * kTileF4;

template <int CBSZ, int ABID>
__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, CBSZ, ABID, 0);
}

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }
__device__ __forceinline__ f32x4 splat(float v) { f32x4 r = {v, v, v, v}; return r; }

// A dependent v_mfma_f32_4x4x1 issues half a pass late (measured: 12.3 instead of 8.2 clocks), so
// every product runs on two accumulators that take turns; the caller adds them at the end.
struct Acc2 {
    f32x4 a, b;
    __device__ __forceinline__ void init(float first) { a = splat(first); b = splat(0.f); }
    __device__ __forceinline__ f32x4 sum() const { return a + b; }
};
// one weight tile, wide layer, narrow (Q) input: input features 4*KG .. 4*KG+3 of the register
template <int KG>
__device__ __forceinline__ void tile_wide_q(Acc2 &acc, float q, f32x4 w) {
    acc.a = mfma4<4, 4 * KG + 0>(q, w.x, acc.a);
    acc.b = mfma4<4, 4 * KG + 1>(q, w.y, acc.b);
    acc.a = mfma4<4, 4 * KG + 2>(q, w.z, acc.a);
    acc.b = mfma4<4, 4 * KG + 3>(q, w.w, acc.b);
}
// one weight tile, wide layer, wide (A) input: features 4*B .. 4*B+3 of the 64-group
template <int B>
__device__ __forceinline__ void tile_wide_a(Acc2 &acc, f32x4 a, f32x4 w) {
    acc.a = mfma4<4, B>(a.x, w.x, acc.a);
    acc.b = mfma4<4, B>(a.y, w.y, acc.b);
    acc.a = mfma4<4, B>(a.z, w.z, acc.a);
    acc.b = mfma4<4, B>(a.w, w.w, acc.b);
}
// one weight tile, narrow layer, wide (A) input: group g covers features 16g + 4*QQ .. +3
template <int QQ>
__device__ __forceinline__ void tile_narrow_a(Acc2 &acc, f32x4 a, f32x4 w) {
    acc.a = mfma4<2, QQ>(a.x, w.x, acc.a);
    acc.b = mfma4<2, QQ>(a.y, w.y, acc.b);
    acc.a = mfma4<2, QQ>(a.z, w.z, acc.a);
    acc.b = mfma4<2, QQ>(a.w, w.w, acc.b);
}
// one weight tile, narrow layer, narrow (Q) input: all 16 features (group g: 4g .. 4g+3)
__device__ __forceinline__ void tile_narrow_q(Acc2 &acc, float q, f32x4 w) {
    acc.a = mfma4<2, 0>(q, w.x, acc.a);
    acc.b = mfma4<2, 1>(q, w.y, acc.b);
    acc.a = mfma4<2, 2>(q, w.z, acc.a);
    acc.b = mfma4<2, 3>(q, w.w, acc.b);
}

__device__ __forceinline__ float dpp_xor1(float v) {  // quad_perm [1, 0, 3, 2]
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_xor2(float v) {  // quad_perm [2, 3, 0, 1]
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
}
// D -> A: register i, lane 4b+j  ->  register j, lane 4b+i
__device__ __forceinline__ f32x4 quad_transpose(f32x4 d, bool odd1, bool odd2) {
    const float x0 = dpp_xor1(d.x), x1 = dpp_xor1(d.y), x2 = dpp_xor1(d.z), x3 = dpp_xor1(d.w);
    const float n0 = odd1 ? x1 : d.x, n1 = odd1 ? d.y : x0;
    const float n2 = odd1 ? x3 : d.z, n3 = odd1 ? d.w : x2;
    const float y0 = dpp_xor2(n0), y1 = dpp_xor2(n1), y2 = dpp_xor2(n2), y3 = dpp_xor2(n3);
    f32x4 r;
    r.x = odd2 ? y2 : n0;
    r.z = odd2 ? n2 : y0;
    r.y = odd2 ? y3 : n1;
    r.w = odd2 ? n3 : y1;
    return r;
}
// narrow accumulator (register i = sample i, four partial sums in the four 16-lane groups) -> P
__device__ __forceinline__ float reduce_to_p(f32x4 acc) {
    // (the results are taken with `auto`: converting the builtin's pair to another vector type
    // makes this compiler read the first element twice)
    const auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc.x), __float_as_uint(acc.y), false, false);
    const float p = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc.z), __float_as_uint(acc.w), false, false);
    const float q = __uint_as_float(b[0]) + __uint_as_float(b[1]);
    const auto c = __builtin_amdgcn_permlane16_swap(__float_as_uint(p), __float_as_uint(q), false, false);
    return __uint_as_float(c[0]) + __uint_as_float(c[1]);
}

// Stream of weight chunks (CH tiles) from global memory through a ring of NBUF LDS buffers.
// NBUF = 3: while chunk c is read from LDS, chunk c+1 already sits in the next buffer and chunk
// c+2 in registers (requested a whole chunk earlier), so neither the L2 round trip nor the LDS
// write is waited for.  NBUF = 2 (when LDS is short): chunk c+1 is in registers.
template <int NBUF>
struct QuadStream {
    static constexpr int kPerThread = kChunkF4 / kThreads;  // 8
    typedef float Regs __attribute__((ext_vector_type(4 * kPerThread)));
    const f32x4 *src;
    f32x4 *buf;
    int total, cur_chunk, cur_buf, tid, rot;
    Regs regs, first[NBUF - 1];  // `first` only lives from start_fetch() to start_commit()

    __device__ __forceinline__ Regs fetch(int chunk) const {
        if (chunk >= total) chunk = total - 1;  // past the end: refetch the last chunk (never used)
        Regs r;
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const f32x4 t = src[(size_t)chunk * kChunkF4 + tid + ((i + rot) & (kPerThread - 1)) * kThreads];
            r[4 * i] = t.x; r[4 * i + 1] = t.y; r[4 * i + 2] = t.z; r[4 * i + 3] = t.w;
        }
        return r;
    }
    __device__ __forceinline__ void commit(Regs r, int b) const {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const f32x4 t = {r[4 * i], r[4 * i + 1], r[4 * i + 2], r[4 * i + 3]};
            buf[b * kChunkF4 + tid + ((i + rot) & (kPerThread - 1)) * kThreads] = t;
        }
    }
    // The first NBUF chunks are requested together at the very start of the kernel (one L2 round
    // trip, hidden behind the set-up of the other LDS tables) and land in LDS before the guide loop.
    // Workgroups walk a chunk's 4 KiB slabs in rotated order so that the compute units of one XCD
    // do not all ask the same L2 channel for the same lines at the same moment.
    __device__ __forceinline__ void start_fetch(const f32x4 *s, f32x4 *b, int n, int t, int rotation) {
        src = s; buf = b; total = n; tid = t; cur_chunk = 0; cur_buf = 0; rot = rotation & (kPerThread - 1);
#pragma unroll
        for (int c = 0; c < NBUF - 1; ++c) first[c] = fetch(c);
        regs = fetch(NBUF - 1);
    }
    __device__ __forceinline__ void start_commit() {  // caller synchronises the workgroup afterwards
#pragma unroll
        for (int c = 0; c < NBUF - 1; ++c) commit(first[c], c);
    }
    __device__ __forceinline__ void advance() {
        ++cur_chunk;
        cur_buf = cur_buf + 1 == NBUF ? 0 : cur_buf + 1;
        if constexpr (NBUF == 3) {
            const int nb = cur_buf + 1 == NBUF ? 0 : cur_buf + 1;  // held chunk cur-2: everyone left it a barrier ago
            commit(regs, nb);
            regs = fetch(cur_chunk + 2);
        } else {
            commit(regs, cur_buf);
            regs = fetch(cur_chunk + 1);
        }
        __syncthreads();
    }
    // The same hand-over in eight pieces, one per 4 KiB slab, for callers that spread it over a
    // chunk's matrix work: slab(i) for every i in 0..7 (any order), then advance_light().
    __device__ __forceinline__ void slab(int i) {
        const int target = cur_buf + NBUF - 1 >= NBUF ? cur_buf - 1 : cur_buf + NBUF - 1;
        const int at = tid + ((i + rot) & (kPerThread - 1)) * kThreads;
        const f32x4 t = {regs[4 * i], regs[4 * i + 1], regs[4 * i + 2], regs[4 * i + 3]};
        buf[target * kChunkF4 + at] = t;
        int chunk = cur_chunk + NBUF;
        if (chunk >= total) chunk = total - 1;
        const f32x4 n = src[(size_t)chunk * kChunkF4 + at];
        regs[4 * i] = n.x; regs[4 * i + 1] = n.y; regs[4 * i + 2] = n.z; regs[4 * i + 3] = n.w;
    }
    __device__ __forceinline__ void advance_light() {
        ++cur_chunk;
        cur_buf = cur_buf + 1 == NBUF ? 0 : cur_buf + 1;
        __syncthreads();
    }
    __device__ __forceinline__ f32x4 tile(int t, int lane) const { return buf[cur_buf * kChunkF4 + t * kTileF4 + lane]; }
};

// use(ic<g>, tiles[4]) for every group of four consecutive tiles.  A SIMD receives LDS data at
// 32 bytes per clock, i.e. one 1 KiB tile in the time its four matrix instructions take, so the
// reads must never be waited for: the tiles of group g+2 are requested (and the request pinned
// in place by scheduling fences) before group g is used -- two groups = 256 clocks of cover.
template <int COUNT, typename LoadF, typename UseG, typename PreG>
__device__ __forceinline__ void for_tile_quads(LoadF &&load, UseG &&use, PreG &&pre) {
    static_assert(COUNT % 4 == 0, "whole groups of four tiles");
    constexpr int kGroups = COUNT / 4;
    f32x4 buf[3][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) buf[0][j] = load(j);
    if constexpr (kGroups > 1) {
#pragma unroll
        for (int j = 0; j < 4; ++j) buf[1][j] = load(4 + j);
    }
    static_for<0, kGroups>([&](auto gc) {
        constexpr int g = decltype(gc)::value;
        if constexpr (g + 2 < kGroups) {
#pragma unroll
            for (int j = 0; j < 4; ++j) buf[(g + 2) % 3][j] = load((g + 2) * 4 + j);
        }
        pre(gc);
        sched_fence();
        use(gc, buf[g % 3]);
        sched_fence();
    });
}
template <int COUNT, typename LoadF, typename UseG>
__device__ __forceinline__ void for_tile_quads(LoadF &&load, UseG &&use) {
    for_tile_quads<COUNT>(load, use, [](auto) {});
}

template <int ZQ, int RG, int HG, int NBUF, bool DBG>
__global__ __launch_bounds__(kThreads) void sample_quad(ChainArgs a) {
    extern __shared__ __align__(16) char lds_raw[];
    constexpr int kCombTiles = 4 * ZQ * RG, kMuTiles = 4 * ZQ * RG, kSigTiles = ZQ * ZQ;
    constexpr int kGuideTiles = kCombTiles + kMuTiles + kSigTiles;
    constexpr int Z16 = 16 * ZQ, R64 = 64 * RG, H64 = 64 * HG;
    constexpr QuadPlan plan = quad_plan(ZQ, HG);
    f32x4 *gw = reinterpret_cast<f32x4 *>(lds_raw);
    f32x4 *ring = gw + kGuideTiles * kTileF4;
    float *ctx = reinterpret_cast<float *>(ring + NBUF * kChunkF4);  // [L][R64]
    float *bias = ctx + a.L * R64;
    const int NG = (a.N + 63) / 64, N64 = NG * 64;
    float *lb_comb = bias, *lb_mu = lb_comb + R64, *lb_sig = lb_mu + Z16;
    float *lb_gate1 = lb_sig + Z16, *lb_gate2 = lb_gate1 + H64, *lb_prop1 = lb_gate2 + Z16;
    float *lb_prop2 = lb_prop1 + H64, *lb_lin = lb_prop2 + Z16, *lb_tscale = lb_lin + Z16;
    float *lb_emean1 = lb_tscale + Z16, *lb_escale1 = lb_emean1 + H64, *lb_emean2 = lb_escale1 + H64;
    float *lb_escale2 = lb_emean2 + N64;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = a.S, Z = a.Z, N = a.N;
    const int s0 = (blockIdx.x * (kThreads / 64) + wave) * 4;  // first sample of this wavefront
    const bool odd1 = lane & 1, odd2 = lane & 2;
    // P layout: lane 16r + k -> feature k of sample s0 + sigma(r)
    const int pk = lane & 15, pr = lane >> 4;
    const int p_smp = s0 + (((pr & 1) << 1) | (pr >> 1));
    const int p_sc = p_smp < S ? p_smp : S - 1;
    // P -> Q: lane 4k + i takes lane 16 sigma(i) + k
    const int qi = lane & 3, qk = lane >> 2;
    const int p2q = 4 * (16 * (((qi & 1) << 1) | (qi >> 1)) + qk);
    auto to_q = [&](float p) {
        return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(p2q, __builtin_bit_cast(int, p)));
    };
    // D layout: register i -> sample s0 + i (clamped: lanes past the end repeat the last sample)
    int d_sc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) d_sc[i] = s0 + i < S ? s0 + i : S - 1;

    // everything the first guide step needs from global memory is requested up front, together
    // with the weight stream's first chunks, so that the round trips overlap
    float zQ[ZQ], eps[ZQ];
#pragma unroll
    for (int zq = 0; zq < ZQ; ++zq) {
        const int fq = zq * 16 + qk, fp = zq * 16 + pk;
        const float z0v = a.z0[fq < Z ? fq : Z - 1];
        const float ev = a.eps_q[(size_t)p_sc * Z + (fp < Z ? fp : Z - 1)];
        zQ[zq] = fq < Z ? z0v : 0.f;
        eps[zq] = fp < Z ? ev : 0.f;
    }
    QuadStream<NBUF> ws;
    ws.start_fetch(reinterpret_cast<const f32x4 *>(a.stream_tiles), ring, a.stream_chunks, tid, blockIdx.x >> 3);
    // Guide weights: small sets stay in registers for all L steps (every wavefront holds all of
    // them: a SIMD receives LDS data no faster than its matrix pipe consumes it, so operands that
    // are reused L times should not come from LDS); larger sets go to LDS.
    constexpr bool kGuideRegs = kGuideTiles <= 20;
    f32x4 gr[kGuideRegs ? kGuideTiles : 1];
    if constexpr (kGuideRegs) {
#pragma unroll
        for (int i = 0; i < kGuideTiles; ++i) gr[i] = reinterpret_cast<const f32x4 *>(a.guide_tiles)[i * kTileF4 + lane];
    }
    // encodings and all biases (and the larger guide weight sets) -> LDS; loads are issued in
    // batches ahead of the stores so that the memory round trips overlap
    {
        if constexpr (!kGuideRegs) {
            const f32x4 *src = reinterpret_cast<const f32x4 *>(a.guide_tiles);
            constexpr int n = kGuideTiles * kTileF4;
            for (int base = 0; base < n; base += 8 * kThreads) {
                f32x4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int i = base + tid + u * kThreads;
                    v[u] = src[i < n ? i : n - 1];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int i = base + tid + u * kThreads;
                    if (i < n) gw[i] = v[u];
                }
            }
        }
        // (1 + h_left + h_right) / 3 per position: the constant part of h_out = (tanh(.) + ...) / 3
        // with tanh written as 1 - 2 r; features past R read as (1 + 0 + 0) / 3, which makes their
        // h_out exactly 0 (tanh(0) = 0)
        const int nc = a.L * R64;
        const int nb = R64 + 6 * Z16 + 4 * H64 + 2 * N64;
        auto load_ctx = [&](int base, float(&f)[8], float(&b)[8]) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = base + tid + u * kThreads;
                const int ic = i < nc ? i : nc - 1;
                const int t = ic / R64, r = ic % R64, rc = r < a.R ? r : a.R - 1;
                f[u] = a.ctx_f[(size_t)t * a.Rp + rc];
                b[u] = a.ctx_b[(size_t)t * a.Rp + rc];
            }
        };
        auto store_ctx = [&](int base, const float(&f)[8], const float(&b)[8]) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = base + tid + u * kThreads;
                if (i < nc) ctx[i] = ((i % R64 < a.R ? f[u] + b[u] : 0.f) + 1.0f) * (1.0f / 3.0f);
            }
        };
        auto load_bias = [&](int base, float(&v)[4]) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + tid + u * kThreads;
                v[u] = a.bias_table[i < nb ? i : nb - 1];
            }
        };
        auto store_bias = [&](int base, const float(&v)[4]) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + tid + u * kThreads;
                if (i < nb) bias[i] = v[u];
            }
        };
        {   // first batch of both tables in one round trip; the common sizes need no second
            float f[8], b[8], v[4];
            load_ctx(0, f, b);
            load_bias(0, v);
            store_ctx(0, f, b);
            store_bias(0, v);
        }
        for (int base = 8 * kThreads; base < nc; base += 8 * kThreads) {
            float f[8], b[8];
            load_ctx(base, f, b);
            store_ctx(base, f, b);
        }
        for (int base = 4 * kThreads; base < nb; base += 4 * kThreads) {
            float v[4];
            load_bias(base, v);
            store_bias(base, v);
        }
    }
    ws.start_commit();
    __syncthreads();
    // guide tile t: comb [zq][kg][og] at 0, mu [zq][ig][q] at kCombTiles, sig [zo][zi] after that
    auto gtile = [&](int t) { return kGuideRegs ? gr[kGuideRegs ? t : 0] : gw[t * kTileF4 + lane]; };

    auto load_p_noise = [&](const float *base, int zq) {  // base -> [S][Z]
        const int f = zq * 16 + pk;
        const float v = base[(size_t)p_sc * Z + (f < Z ? f : Z - 1)];
        return f < Z ? v : 0.f;
    };
    auto store_p = [&](float *dst, int zq, float v) {  // dst [S][Z]
        if (!DBG || !dst) return;
        const int f = zq * 16 + pk;
        if (p_smp < S && f < Z) dst[(size_t)p_smp * Z + f] = v;
    };

    float b_comb[RG], b_mu[ZQ], b_sig[ZQ];
#pragma unroll
    for (int og = 0; og < RG; ++og) b_comb[og] = lb_comb[og * 64 + lane];
#pragma unroll
    for (int zq = 0; zq < ZQ; ++zq) { b_mu[zq] = lb_mu[zq * 16 + pk]; b_sig[zq] = lb_sig[zq * 16 + pk]; }

    // ---- guide chain ------------------------------------------------------------
    float zP[ZQ];
#pragma unroll
    for (int zq = 0; zq < ZQ; ++zq) zP[zq] = 0.f;
    for (int t = 0; t < a.L; ++t) {
        float eps_next[ZQ];  // next step's noise is fetched while this step computes
        const int tn = t + 1 < a.L ? t + 1 : t;
#pragma unroll
        for (int zq = 0; zq < ZQ; ++zq) eps_next[zq] = load_p_noise(a.eps_q + (size_t)tn * S * Z, zq);
        // combiner: h_out = (tanh(W_c z + b) + h_left + h_right) / 3, tiles [zq][kg][og]
        Acc2 acc[RG];
#pragma unroll
        for (int og = 0; og < RG; ++og) acc[og].init(b_comb[og]);
        static_for<0, ZQ>([&](auto zc) {
            constexpr int zq = decltype(zc)::value;
            static_for<0, 4>([&](auto kc) {
                constexpr int kg = decltype(kc)::value;
#pragma unroll
                for (int og = 0; og < RG; ++og)
                    tile_wide_q<kg>(acc[og], zQ[zq], gtile((zq * 4 + kg) * RG + og));
            });
        });
        f32x4 hA[RG];
#pragma unroll
        for (int og = 0; og < RG; ++og) {
            const float c = ctx[t * R64 + og * 64 + lane];
            const f32x4 v = acc[og].sum();
            f32x4 h;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[i] = fast_rcp(__expf(2.0f * v[i]) + 1.0f) * (-2.0f / 3.0f) + c;
            hA[og] = quad_transpose(h, odd1, odd2);
        }
        // mu = W_mu h_out + b, tiles [zq][ig][q]; two accumulators in turn
        float muP[ZQ], muQ[ZQ];
        static_for<0, ZQ>([&](auto zc) {
            constexpr int zq = decltype(zc)::value;
            Acc2 n;
            n.init(0.f);
            static_for<0, RG>([&](auto ic) {
                constexpr int ig = decltype(ic)::value;
                constexpr int w = kCombTiles + (zq * RG + ig) * 4;
                tile_narrow_a<0>(n, hA[ig], gtile(w + 0));
                tile_narrow_a<1>(n, hA[ig], gtile(w + 1));
                tile_narrow_a<2>(n, hA[ig], gtile(w + 2));
                tile_narrow_a<3>(n, hA[ig], gtile(w + 3));
            });
            muP[zq] = reduce_to_p(n.sum()) + b_mu[zq];
            muQ[zq] = to_q(muP[zq]);
        });
        // sigma = softplus(W_sigma mu + b), z = mu + sigma eps, tiles [zo][zi]
#pragma unroll
        for (int zo = 0; zo < ZQ; ++zo) {
            Acc2 n;
            n.init(0.f);
#pragma unroll
            for (int zi = 0; zi < ZQ; ++zi) tile_narrow_q(n, muQ[zi], gtile(kCombTiles + kMuTiles + zo * ZQ + zi));
            const float pre = reduce_to_p(n.sum()) + b_sig[zo];
            zP[zo] = muP[zo] + softplus_f(pre) * eps[zo];
            eps[zo] = eps_next[zo];
        }
#pragma unroll
        for (int zq = 0; zq < ZQ; ++zq) zQ[zq] = to_q(zP[zq]);
    }
#pragma unroll
    for (int zq = 0; zq < ZQ; ++zq) store_p(a.z_last, zq, zP[zq]);

    // ---- streamed part: transition, then emission --------------------------------
    int chunk_now = 0;  // compile-time after unrolling: chunk the stream is positioned at
    auto seek = [&](int chunk) {  // layers are laid out so that none straddles a chunk
        while (chunk_now < chunk) { ws.advance(); ++chunk_now; }
    };

    // out (D, HG groups) = W x + b for a narrow -> wide layer at stream position `pos`, tiles [zq][kg][og]
    auto wide_from_q = [&](f32x4(&out)[HG], const float *tab, const float(&x)[ZQ], int pos) {
        seek(pos / CH);
        const int base = pos % CH;
        Acc2 acc[HG];
#pragma unroll
        for (int og = 0; og < HG; ++og) acc[og].init(tab[og * 64 + lane]);
        // groups of four tiles: (zq, kg) major, og minor
        for_tile_quads<4 * ZQ * HG>([&](int i) { return ws.tile(base + i, lane); },
                                    [&](auto gc, const f32x4(&tl)[4]) {
                                        constexpr int g = decltype(gc)::value;
                                        static_for<0, 4>([&](auto jc) {
                                            constexpr int idx = g * 4 + decltype(jc)::value;
                                            constexpr int og = idx % HG, kk = idx / HG;  // kk = zq * 4 + kg
                                            tile_wide_q<kk % 4>(acc[og], x[kk / 4], tl[decltype(jc)::value]);
                                        });
                                    });
#pragma unroll
        for (int og = 0; og < HG; ++og) out[og] = acc[og].sum();
    };
    // out (P, per zq) = W h + b for a wide -> narrow layer, tiles [zq][ig][q]
    auto narrow_from_a = [&](float(&out)[ZQ], const float *tab, const f32x4(&x)[HG], int pos) {
        seek(pos / CH);
        const int base = pos % CH;
        Acc2 n[ZQ];
#pragma unroll
        for (int zq = 0; zq < ZQ; ++zq) n[zq].init(0.f);
        for_tile_quads<4 * ZQ * HG>([&](int i) { return ws.tile(base + i, lane); },
                                    [&](auto gc, const f32x4(&tl)[4]) {
                                        constexpr int g = decltype(gc)::value;
                                        constexpr int zq = g / HG, ig = g % HG;
                                        tile_narrow_a<0>(n[zq], x[ig], tl[0]);
                                        tile_narrow_a<1>(n[zq], x[ig], tl[1]);
                                        tile_narrow_a<2>(n[zq], x[ig], tl[2]);
                                        tile_narrow_a<3>(n[zq], x[ig], tl[3]);
                                    });
#pragma unroll
        for (int zq = 0; zq < ZQ; ++zq) out[zq] = reduce_to_p(n[zq].sum()) + tab[zq * 16 + pk];
    };
    // out (P) = W x + b for a narrow -> narrow layer, tiles [zo][zi] (padded to a multiple of four)
    auto small_layer = [&](float(&out)[ZQ], const float *tab, const float(&x)[ZQ], int pos) {
        seek(pos / CH);
        const int base = pos % CH;
#pragma unroll
        for (int zo = 0; zo < ZQ; ++zo) {
            Acc2 n;
            n.init(0.f);
#pragma unroll
            for (int zi = 0; zi < ZQ; ++zi) tile_narrow_q(n, x[zi], ws.tile(base + zo * ZQ + zi, lane));
            out[zo] = reduce_to_p(n.sum()) + tab[zo * 16 + pk];
        }
    };
    auto to_a = [&](f32x4(&dst)[HG], const f32x4(&src)[HG], bool relu) {
#pragma unroll
        for (int og = 0; og < HG; ++og) {
            f32x4 v = src[og];
            if (relu) {
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = fmaxf(v[i], 0.f);
            }
            dst[og] = quad_transpose(v, odd1, odd2);
        }
    };

    float znQ[ZQ];
    {
        f32x4 d[HG], hidG[HG], hidP[HG];
        float lin[ZQ], g[ZQ], prop[ZQ], G[ZQ], rGQ[ZQ], pre[ZQ];
        wide_from_q(d, lb_gate1, zQ, plan.gate1);
        to_a(hidG, d, true);
        wide_from_q(d, lb_prop1, zQ, plan.prop1);
        to_a(hidP, d, true);
        small_layer(lin, lb_lin, zQ, plan.lin);
        narrow_from_a(g, lb_gate2, hidG, plan.gate2);
        narrow_from_a(prop, lb_prop2, hidP, plan.prop2);
#pragma unroll
        for (int zq = 0; zq < ZQ; ++zq) {
            const float gate = sigmoid_f(g[zq]);
            G[zq] = (1.f - gate) * lin[zq] + gate * prop[zq];
            rGQ[zq] = to_q(fmaxf(G[zq], 0.f));
        }
        small_layer(pre, lb_tscale, rGQ, plan.tscale);
#pragma unroll
        for (int zq = 0; zq < ZQ; ++zq) {
            const float e = load_p_noise(a.eps_z, zq);
            float zn = G[zq] + softplus_f(pre[zq]) * e;
            if (zq * 16 + pk >= Z) zn = 0.f;
            store_p(a.z_next_dbg, zq, zn);
            znQ[zq] = to_q(zn);
        }
    }

    // emission: hidden layer of the mean
    f32x4 h1A[HG];
    {
        f32x4 d[HG];
        wide_from_q(d, lb_emean1, znQ, plan.emean1);
        to_a(h1A, d, a.emit_mean_act != 0);
    }
    seek(plan.head_chunks);

    // mean, 64 workers at a time, each group folded into the scale network's hidden layer at once:
    // per group og the stream holds HG*16 tiles of the mean's second layer (row group og), then
    // HG*16 tiles of the scale network's first layer (column group og)
    constexpr int kSegs = HG < 2 ? 1 : HG / 2;  // 32-tile chunks per 16*HG tiles
    constexpr int kSegTiles = HG < 2 ? 16 : 32;
    Acc2 h2[HG];
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) h2[hg].init(lb_escale1[hg * 64 + lane]);
    float *sink = a.sink + tid;
    for (int og = 0; og < NG; ++og) {
        const int col = og * 64 + lane;
        Acc2 macc;
        macc.init(lb_emean2[col]);
        static_for<0, kSegs>([&](auto sc) {
            constexpr int seg = decltype(sc)::value;
            for_tile_quads<kSegTiles>([&](int i) { return ws.tile(i, lane); },
                                      [&](auto gc, const f32x4(&tl)[4]) {
                                          constexpr int t0 = seg * kSegTiles + decltype(gc)::value * 4;  // tile = ig*16 + b
                                          tile_wide_a<(t0 + 0) % 16>(macc, h1A[(t0 + 0) / 16], tl[0]);
                                          tile_wide_a<(t0 + 1) % 16>(macc, h1A[(t0 + 1) / 16], tl[1]);
                                          tile_wide_a<(t0 + 2) % 16>(macc, h1A[(t0 + 2) / 16], tl[2]);
                                          tile_wide_a<(t0 + 3) % 16>(macc, h1A[(t0 + 3) / 16], tl[3]);
                                      },
                                      [&](auto gc) { ws.slab(decltype(gc)::value); });  // HG = 1: slabs 0..3
            if constexpr (HG >= 2) ws.advance_light();
        });
        const f32x4 mean = macc.sum();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float *dst = col < N ? a.mean + (size_t)d_sc[i] * a.ld_mean + col : sink;
            *dst = mean[i];
        }
        const f32x4 mA = quad_transpose(mean, odd1, odd2);
        // scale network, first layer: h2[hg] += W[64 hg + l][64 og + 4 b + j] mean, tiles [b][hg]
        static_for<0, kSegs>([&](auto sc) {
            constexpr int seg = decltype(sc)::value;
            constexpr int off = HG < 2 ? 16 : 0;  // HG = 1: both halves share one chunk
            for_tile_quads<kSegTiles>([&](int i) { return ws.tile(off + i, lane); },
                                      [&](auto gc, const f32x4(&tl)[4]) {
                                          constexpr int t0 = seg * kSegTiles + decltype(gc)::value * 4;  // tile = b*HG + hg
                                          tile_wide_a<(t0 + 0) / HG>(h2[(t0 + 0) % HG], mA, tl[0]);
                                          tile_wide_a<(t0 + 1) / HG>(h2[(t0 + 1) % HG], mA, tl[1]);
                                          tile_wide_a<(t0 + 2) / HG>(h2[(t0 + 2) % HG], mA, tl[2]);
                                          tile_wide_a<(t0 + 3) / HG>(h2[(t0 + 3) % HG], mA, tl[3]);
                                      },
                                      [&](auto gc) { ws.slab((HG < 2 ? 4 : 0) + decltype(gc)::value); });
            if constexpr (HG >= 2) ws.advance_light();
        });
        if constexpr (HG < 2) ws.advance_light();
    }
    f32x4 h2A[HG];
    {
        f32x4 d[HG];
#pragma unroll
        for (int hg = 0; hg < HG; ++hg) d[hg] = h2[hg].sum();
        to_a(h2A, d, true);
    }

    // scale, draw, back to seconds: per group og HG*16 tiles of the scale network's second layer
    const float scale = a.ctl->scale;
    for (int og = 0; og < NG; ++og) {
        const int col = og * 64 + lane;
        const int colc = col < N ? col : N - 1;
        f32x4 e, m;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            e[i] = a.eps_x[(size_t)d_sc[i] * N + colc];
            m[i] = a.mean[(size_t)d_sc[i] * a.ld_mean + colc];
        }
        Acc2 pacc;
        pacc.init(lb_escale2[col]);
        static_for<0, kSegs>([&](auto sc) {
            constexpr int seg = decltype(sc)::value;
            for_tile_quads<kSegTiles>([&](int i) { return ws.tile(i, lane); },
                                      [&](auto gc, const f32x4(&tl)[4]) {
                                          constexpr int t0 = seg * kSegTiles + decltype(gc)::value * 4;
                                          tile_wide_a<(t0 + 0) % 16>(pacc, h2A[(t0 + 0) / 16], tl[0]);
                                          tile_wide_a<(t0 + 1) % 16>(pacc, h2A[(t0 + 1) / 16], tl[1]);
                                          tile_wide_a<(t0 + 2) % 16>(pacc, h2A[(t0 + 2) / 16], tl[2]);
                                          tile_wide_a<(t0 + 3) % 16>(pacc, h2A[(t0 + 3) / 16], tl[3]);
                                      },
                                      [&](auto gc) {
                                          constexpr int g = decltype(gc)::value;
                                          if constexpr (HG < 2) { ws.slab(2 * g); ws.slab(2 * g + 1); }  // 4 groups per chunk
                                          else ws.slab(g);
                                      });
            ws.advance_light();
        });
        const f32x4 pre = pacc.sum();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float sd = softplus_f(pre[i]);
            const float x = (m[i] + sd * e[i]) * scale;
            float *dst = col < N ? a.out_samples + (size_t)d_sc[i] * N + col : sink;
            *dst = x;
            if constexpr (DBG) {
                if (col < N && s0 + i < S) {
                    if (a.out_mean_dbg) a.out_mean_dbg[(size_t)(s0 + i) * N + col] = m[i];
                    if (a.out_sd_dbg) a.out_sd_dbg[(size_t)(s0 + i) * N + col] = sd;
                }
            }
        }
    }
}

template <int ZQ, int RG, int HG, int NBUF>
size_t quad_lds_bytes(int L, int N) {
    const size_t n64 = (size_t)((N + 63) / 64) * 64;
    const size_t bias_floats = 64 * RG + 6 * 16 * ZQ + 4 * 64 * HG + 2 * n64;
    return (size_t)(8 * ZQ * RG + ZQ * ZQ + NBUF * CH) * kTileF4 * 16 + ((size_t)L * 64 * RG + bias_floats) * 4;
}

template <int ZQ, int RG, int HG, int NBUF, bool DBG>
int launch_variant(const ChainArgs &a, size_t lds, hipStream_t stream) {
    static size_t raised = 0;  // largest LDS size the attribute has been set to
    if (lds > raised) {
        DKF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(sample_quad<ZQ, RG, HG, NBUF, DBG>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        raised = lds;
    }
    const int per_block = (kThreads / 64) * 4;
    const dim3 grid((a.S + per_block - 1) / per_block);
    hipLaunchKernelGGL((sample_quad<ZQ, RG, HG, NBUF, DBG>), grid, dim3(kThreads), lds, stream, a);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

template <int ZQ, int RG, int HG>
int launch_one(const ChainArgs &a, hipStream_t stream) {
    const bool dbg = a.z_last || a.z_next_dbg || a.out_mean_dbg || a.out_sd_dbg;
    size_t lds = quad_lds_bytes<ZQ, RG, HG, 3>(a.L, a.N);
    if (lds <= 160 * 1024)
        return dbg ? launch_variant<ZQ, RG, HG, 3, true>(a, lds, stream) : launch_variant<ZQ, RG, HG, 3, false>(a, lds, stream);
    lds = quad_lds_bytes<ZQ, RG, HG, 2>(a.L, a.N);
    if (lds > 160 * 1024) return DKF_EUNSUPPORTED;
    return dbg ? launch_variant<ZQ, RG, HG, 2, true>(a, lds, stream) : launch_variant<ZQ, RG, HG, 2, false>(a, lds, stream);
}

}  // namespace

bool quad_supported(int Z, int R, int H, int L, int N) {
    const int zq = (Z + 15) / 16, rg = (R + 63) / 64, hg = (H + 63) / 64;
    size_t lds;
    if (zq == 1 && rg == 1 && hg == 1) lds = quad_lds_bytes<1, 1, 1, 2>(L, N);
    else if (zq == 1 && rg == 2 && hg == 2) lds = quad_lds_bytes<1, 2, 2, 2>(L, N);
    else if (zq == 2 && rg == 4 && hg == 4) lds = quad_lds_bytes<2, 4, 4, 2>(L, N);
    else return false;
    return lds <= 160 * 1024 && N >= 1 && Z >= 1;
}

int launch_quad(const ChainArgs &a, hipStream_t stream) {
    StageTimer timer(kStageSampler, stream);
    const int zq = (a.Z + 15) / 16, rg = (a.R + 63) / 64, hg = (a.H + 63) / 64;
    if (zq == 1 && rg == 1 && hg == 1) return launch_one<1, 1, 1>(a, stream);
    if (zq == 1 && rg == 2 && hg == 2) return launch_one<1, 2, 2>(a, stream);
    if (zq == 2 && rg == 4 && hg == 4) return launch_one<2, 4, 4>(a, stream);
    return DKF_EUNSUPPORTED;
}

}  // namespace dkf
