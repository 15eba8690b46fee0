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

// one weight tile, wide layer, narrow (Q) input: input features 4*KG .. 4*KG+3 of the register
template <int KG>
__device__ __forceinline__ void tile_wide_q(f32x4 &acc, float q, f32x4 w) {
    acc = mfma4<4, 4 * KG + 0>(q, w.x, acc);
    acc = mfma4<4, 4 * KG + 1>(q, w.y, acc);
    acc = mfma4<4, 4 * KG + 2>(q, w.z, acc);
    acc = mfma4<4, 4 * KG + 3>(q, w.w, acc);
}
// one weight tile, wide layer, wide (A) input: features 4*B .. 4*B+3 of the 64-group
template <int B>
__device__ __forceinline__ void tile_wide_a(f32x4 &acc, f32x4 a, f32x4 w) {
    acc = mfma4<4, B>(a.x, w.x, acc);
    acc = mfma4<4, B>(a.y, w.y, acc);
    acc = mfma4<4, B>(a.z, w.z, acc);
    acc = mfma4<4, B>(a.w, w.w, acc);
}
// one weight tile, narrow layer, wide (A) input: group g covers features 16g + 4*QQ .. +3
template <int QQ>
__device__ __forceinline__ void tile_narrow_a(f32x4 &acc, f32x4 a, f32x4 w) {
    acc = mfma4<2, QQ>(a.x, w.x, acc);
    acc = mfma4<2, QQ>(a.y, w.y, acc);
    acc = mfma4<2, QQ>(a.z, w.z, acc);
    acc = mfma4<2, QQ>(a.w, w.w, acc);
}
// one weight tile, narrow layer, narrow (Q) input: all 16 features (group g: 4g .. 4g+3)
__device__ __forceinline__ void tile_narrow_q(f32x4 &acc, float q, f32x4 w) {
    acc = mfma4<2, 0>(q, w.x, acc);
    acc = mfma4<2, 1>(q, w.y, acc);
    acc = mfma4<2, 2>(q, w.z, acc);
    acc = mfma4<2, 3>(q, w.w, acc);
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
    int total, cur_chunk, cur_buf, tid;
    Regs regs;

    __device__ __forceinline__ Regs fetch(int chunk) const {
        if (chunk >= total) chunk = total - 1;  // past the end: refetch the last chunk (never used)
        Regs r;
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const f32x4 t = src[(size_t)chunk * kChunkF4 + tid + i * kThreads];
            r[4 * i] = t.x; r[4 * i + 1] = t.y; r[4 * i + 2] = t.z; r[4 * i + 3] = t.w;
        }
        return r;
    }
    __device__ __forceinline__ void commit(Regs r, int b) const {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const f32x4 t = {r[4 * i], r[4 * i + 1], r[4 * i + 2], r[4 * i + 3]};
            buf[b * kChunkF4 + tid + i * kThreads] = t;
        }
    }
    __device__ __forceinline__ void start(const f32x4 *s, f32x4 *b, int n, int t) {
        src = s; buf = b; total = n; tid = t; cur_chunk = 0; cur_buf = 0;
        regs = fetch(0);
        commit(regs, 0);
        if constexpr (NBUF == 3) {
            regs = fetch(1);
            commit(regs, 1);
            regs = fetch(2);
        } else {
            regs = fetch(1);
        }
        __syncthreads();
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
    __device__ __forceinline__ f32x4 tile(int t, int lane) const { return buf[cur_buf * kChunkF4 + t * kTileF4 + lane]; }
};

// use(ic<g>, tiles[4]) for every group of four consecutive tiles; the next group's tiles are
// read from LDS while the current group feeds the matrix cores.
template <int COUNT, typename LoadF, typename UseG>
__device__ __forceinline__ void for_tile_quads(LoadF &&load, UseG &&use) {
    static_assert(COUNT % 4 == 0, "whole groups of four tiles");
    constexpr int kGroups = COUNT / 4;
    f32x4 buf[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) buf[0][j] = load(j);
    static_for<0, kGroups>([&](auto gc) {
        constexpr int g = decltype(gc)::value;
        if constexpr (g + 1 < kGroups) {
#pragma unroll
            for (int j = 0; j < 4; ++j) buf[(g + 1) & 1][j] = load((g + 1) * 4 + j);
        }
        use(gc, buf[g & 1]);
        sched_fence();
    });
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

    // guide weights, encodings and all biases -> LDS
    {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(a.guide_tiles);
        for (int i = tid; i < kGuideTiles * kTileF4; i += kThreads) gw[i] = src[i];
        // (1 + h_left + h_right) / 3 per position: the constant part of h_out = (tanh(.) + ...) / 3
        // with tanh written as 1 - 2 r; features past R read as (1 + 0 + 0) / 3, which makes their
        // h_out exactly 0 (tanh(0) = 0)
        for (int i = tid; i < a.L * R64; i += kThreads) {
            const int t = i / R64, r = i % R64;
            const float f = r < a.R ? a.ctx_f[(size_t)t * a.Rp + r] + a.ctx_b[(size_t)t * a.Rp + r] : 0.f;
            ctx[i] = (f + 1.0f) * (1.0f / 3.0f);
        }
        const int nb = R64 + 6 * Z16 + 4 * H64 + 2 * N64;
        for (int i = tid; i < nb; i += kThreads) bias[i] = a.bias_table[i];
    }
    __syncthreads();
    const f32x4 *w_comb = gw;                 // [zq][kg][og]
    const f32x4 *w_mu = gw + kCombTiles * kTileF4;  // [zq][ig][q]
    const f32x4 *w_sig = w_mu + kMuTiles * kTileF4; // [zo][zi]

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

    float zQ[ZQ];
#pragma unroll
    for (int zq = 0; zq < ZQ; ++zq) {
        const int f = zq * 16 + qk;
        zQ[zq] = f < Z ? a.z0[f] : 0.f;
    }
    float b_comb[RG], b_mu[ZQ], b_sig[ZQ];
#pragma unroll
    for (int og = 0; og < RG; ++og) b_comb[og] = lb_comb[og * 64 + lane];
#pragma unroll
    for (int zq = 0; zq < ZQ; ++zq) { b_mu[zq] = lb_mu[zq * 16 + pk]; b_sig[zq] = lb_sig[zq * 16 + pk]; }

    // ---- guide chain ------------------------------------------------------------
    float zP[ZQ], eps[ZQ];
#pragma unroll
    for (int zq = 0; zq < ZQ; ++zq) { eps[zq] = load_p_noise(a.eps_q, zq); zP[zq] = 0.f; }
    for (int t = 0; t < a.L; ++t) {
        float eps_next[ZQ];  // next step's noise is fetched while this step computes
        const int tn = t + 1 < a.L ? t + 1 : t;
#pragma unroll
        for (int zq = 0; zq < ZQ; ++zq) eps_next[zq] = load_p_noise(a.eps_q + (size_t)tn * S * Z, zq);
        // combiner: h_out = (tanh(W_c z + b) + h_left + h_right) / 3, tiles [zq][kg][og]
        f32x4 acc[RG];
#pragma unroll
        for (int og = 0; og < RG; ++og) acc[og] = splat(b_comb[og]);
        static_for<0, ZQ>([&](auto zc) {
            constexpr int zq = decltype(zc)::value;
            static_for<0, 4>([&](auto kc) {
                constexpr int kg = decltype(kc)::value;
#pragma unroll
                for (int og = 0; og < RG; ++og)
                    tile_wide_q<kg>(acc[og], zQ[zq], w_comb[((zq * 4 + kg) * RG + og) * kTileF4 + lane]);
            });
        });
        f32x4 hA[RG];
#pragma unroll
        for (int og = 0; og < RG; ++og) {
            const float c = ctx[t * R64 + og * 64 + lane];
            f32x4 h;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[i] = fast_rcp(__expf(2.0f * acc[og][i]) + 1.0f) * (-2.0f / 3.0f) + c;
            hA[og] = quad_transpose(h, odd1, odd2);
        }
        // mu = W_mu h_out + b, tiles [zq][ig][q]; two accumulators in turn
        float muP[ZQ], muQ[ZQ];
        static_for<0, ZQ>([&](auto zc) {
            constexpr int zq = decltype(zc)::value;
            f32x4 n0 = splat(0.f), n1 = splat(0.f);
            static_for<0, RG>([&](auto ic) {
                constexpr int ig = decltype(ic)::value;
                const f32x4 *w = w_mu + ((zq * RG + ig) * 4) * kTileF4 + lane;
                tile_narrow_a<0>(n0, hA[ig], w[0 * kTileF4]);
                tile_narrow_a<1>(n1, hA[ig], w[1 * kTileF4]);
                tile_narrow_a<2>(n0, hA[ig], w[2 * kTileF4]);
                tile_narrow_a<3>(n1, hA[ig], w[3 * kTileF4]);
            });
            muP[zq] = reduce_to_p(n0 + n1) + b_mu[zq];
            muQ[zq] = to_q(muP[zq]);
        });
        // sigma = softplus(W_sigma mu + b), z = mu + sigma eps, tiles [zo][zi]
#pragma unroll
        for (int zo = 0; zo < ZQ; ++zo) {
            f32x4 n = splat(0.f);
#pragma unroll
            for (int zi = 0; zi < ZQ; ++zi) tile_narrow_q(n, muQ[zi], w_sig[(zo * ZQ + zi) * kTileF4 + lane]);
            const float pre = reduce_to_p(n) + b_sig[zo];
            zP[zo] = muP[zo] + softplus_f(pre) * eps[zo];
            eps[zo] = eps_next[zo];
        }
#pragma unroll
        for (int zq = 0; zq < ZQ; ++zq) zQ[zq] = to_q(zP[zq]);
    }
#pragma unroll
    for (int zq = 0; zq < ZQ; ++zq) store_p(a.z_last, zq, zP[zq]);

    // ---- streamed part: transition, then emission --------------------------------
    QuadStream<NBUF> ws;
    ws.start(reinterpret_cast<const f32x4 *>(a.stream_tiles), ring, a.stream_chunks, tid);
    int chunk_now = 0;  // compile-time after unrolling: chunk the stream is positioned at
    auto seek = [&](int chunk) {  // layers are laid out so that none straddles a chunk
        while (chunk_now < chunk) { ws.advance(); ++chunk_now; }
    };

    // out (D, HG groups) = W x + b for a narrow -> wide layer at stream position `pos`, tiles [zq][kg][og]
    auto wide_from_q = [&](f32x4(&out)[HG], const float *tab, const float(&x)[ZQ], int pos) {
        seek(pos / CH);
        const int base = pos % CH;
#pragma unroll
        for (int og = 0; og < HG; ++og) out[og] = splat(tab[og * 64 + lane]);
        // groups of four tiles: (zq, kg) major, og minor
        for_tile_quads<4 * ZQ * HG>([&](int i) { return ws.tile(base + i, lane); },
                                    [&](auto gc, const f32x4(&tl)[4]) {
                                        constexpr int g = decltype(gc)::value;
                                        static_for<0, 4>([&](auto jc) {
                                            constexpr int idx = g * 4 + decltype(jc)::value;
                                            constexpr int og = idx % HG, kk = idx / HG;  // kk = zq * 4 + kg
                                            tile_wide_q<kk % 4>(out[og], x[kk / 4], tl[decltype(jc)::value]);
                                        });
                                    });
    };
    // out (P, per zq) = W h + b for a wide -> narrow layer, tiles [zq][ig][q]
    auto narrow_from_a = [&](float(&out)[ZQ], const float *tab, const f32x4(&x)[HG], int pos) {
        seek(pos / CH);
        const int base = pos % CH;
        f32x4 n0[ZQ], n1[ZQ];
#pragma unroll
        for (int zq = 0; zq < ZQ; ++zq) n0[zq] = n1[zq] = splat(0.f);
        for_tile_quads<4 * ZQ * HG>([&](int i) { return ws.tile(base + i, lane); },
                                    [&](auto gc, const f32x4(&tl)[4]) {
                                        constexpr int g = decltype(gc)::value;
                                        constexpr int zq = g / HG, ig = g % HG;
                                        tile_narrow_a<0>(n0[zq], x[ig], tl[0]);
                                        tile_narrow_a<1>(n1[zq], x[ig], tl[1]);
                                        tile_narrow_a<2>(n0[zq], x[ig], tl[2]);
                                        tile_narrow_a<3>(n1[zq], x[ig], tl[3]);
                                    });
#pragma unroll
        for (int zq = 0; zq < ZQ; ++zq) out[zq] = reduce_to_p(n0[zq] + n1[zq]) + tab[zq * 16 + pk];
    };
    // out (P) = W x + b for a narrow -> narrow layer, tiles [zo][zi] (padded to a multiple of four)
    auto small_layer = [&](float(&out)[ZQ], const float *tab, const float(&x)[ZQ], int pos) {
        seek(pos / CH);
        const int base = pos % CH;
#pragma unroll
        for (int zo = 0; zo < ZQ; ++zo) {
            f32x4 n = splat(0.f);
#pragma unroll
            for (int zi = 0; zi < ZQ; ++zi) tile_narrow_q(n, x[zi], ws.tile(base + zo * ZQ + zi, lane));
            out[zo] = reduce_to_p(n) + tab[zo * 16 + pk];
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
    f32x4 h2[HG];
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) h2[hg] = splat(lb_escale1[hg * 64 + lane]);
    float *sink = a.sink + tid;
    for (int og = 0; og < NG; ++og) {
        const int col = og * 64 + lane;
        f32x4 m0 = splat(lb_emean2[col]), m1 = splat(0.f);
        static_for<0, kSegs>([&](auto sc) {
            constexpr int seg = decltype(sc)::value;
            for_tile_quads<kSegTiles>([&](int i) { return ws.tile(i, lane); },
                                      [&](auto gc, const f32x4(&tl)[4]) {
                                          constexpr int t0 = seg * kSegTiles + decltype(gc)::value * 4;  // tile = ig*16 + b
                                          tile_wide_a<(t0 + 0) % 16>(m0, h1A[(t0 + 0) / 16], tl[0]);
                                          tile_wide_a<(t0 + 1) % 16>(m1, h1A[(t0 + 1) / 16], tl[1]);
                                          tile_wide_a<(t0 + 2) % 16>(m0, h1A[(t0 + 2) / 16], tl[2]);
                                          tile_wide_a<(t0 + 3) % 16>(m1, h1A[(t0 + 3) / 16], tl[3]);
                                      });
            if constexpr (HG >= 2) ws.advance();
        });
        const f32x4 mean = m0 + m1;
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
                                      });
            if constexpr (HG >= 2) ws.advance();
        });
        if constexpr (HG < 2) ws.advance();
    }
    f32x4 h2A[HG];
    to_a(h2A, h2, true);

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
        f32x4 p0 = splat(lb_escale2[col]), p1 = splat(0.f);
        static_for<0, kSegs>([&](auto sc) {
            constexpr int seg = decltype(sc)::value;
            for_tile_quads<kSegTiles>([&](int i) { return ws.tile(i, lane); },
                                      [&](auto gc, const f32x4(&tl)[4]) {
                                          constexpr int t0 = seg * kSegTiles + decltype(gc)::value * 4;
                                          tile_wide_a<(t0 + 0) % 16>(p0, h2A[(t0 + 0) / 16], tl[0]);
                                          tile_wide_a<(t0 + 1) % 16>(p1, h2A[(t0 + 1) / 16], tl[1]);
                                          tile_wide_a<(t0 + 2) % 16>(p0, h2A[(t0 + 2) / 16], tl[2]);
                                          tile_wide_a<(t0 + 3) % 16>(p1, h2A[(t0 + 3) / 16], tl[3]);
                                      });
            ws.advance();
        });
        const f32x4 pre = p0 + p1;
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
