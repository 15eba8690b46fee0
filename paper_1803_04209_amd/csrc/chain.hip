// Posterior-predictive sampling as one register-chained kernel (Sec. 3.1.3):
// guide trajectories z_1..z_L, the gated transition draw z_{T+1} and the
// emission draw x_{T+1}, for 16 samples per wavefront.
//
// Every layer is computed transposed, Y^T = W X^T, with
// v_mfma_f32_16x16x4_f32: the weights are the A operand (16 output features x
// 4 input features per instruction), the activations the B operand (4 input
// features x 16 samples).  Lane l of the result holds output features
// 4*(l/16)+v, v = 0..3, of sample l%16 -- exactly the B-operand placement the
// next layer needs (instruction v of a 16-feature block consumes register v).
// So activations never leave registers between layers, wavefronts never
// exchange data, and the only barriers are those of the weight stream.
//
// Weights: the three guide matrices stay in LDS for all L steps; everything
// after the guide loop (transition, emission) is used once per wavefront and
// is streamed from L2 through a double-buffered LDS ring, in a chunk order
// laid down when the weights are loaded (ChainPack), so that the four
// wavefronts of a workgroup share every fetch.  The scale network's first
// layer is folded with the mean's output layer when the weights are loaded, so
// both hidden vectors are known before the first N-wide product and mean and
// scale of a 16-worker block are produced, and drawn from, together.
#include "common.h"
#include "mfma_tile.h"
#include "mfma16.h"

namespace dkf {
namespace {

constexpr int kThreads = 256;
using AccN = Acc<1>;
constexpr int kTileF4 = 64;  // float4 per weight tile (one per lane)

// Stream of weight chunks (CH tiles each) from global memory through a two-buffer LDS ring, moved
// by global_load_lds_dwordx4: a wavefront's instruction carries one 1 KiB tile (16 bytes per lane,
// consecutive lanes to consecutive LDS addresses, which is the tile's layout) from L2 into LDS
// without passing through registers, so a chunk costs each wavefront CH / 4 load instructions and
// nothing else -- no LDS stores, no staging registers.  While chunk c is consumed, chunk c + 1 is
// on its way into the other buffer (every wavefront was done with that one at the barrier that ended
// chunk c - 1): its load instructions are handed out between the groups of chunk c's matrix
// instructions (spread), whose shadow hides their issue, and next() at the end of chunk c waits for
// the wavefront's own requests (they count in vmcnt like any load; the compiler does not connect
// them with the LDS reads that follow, hence the explicit wait) before the barrier that makes all
// of them visible.  A chunk is sized so that its matrix work outlasts an L2 round trip.
template <int CH>
struct WeightStream {
    static constexpr int kChunkF4 = CH * kTileF4;
    static constexpr int kTilesPerWave = CH / (kThreads / 64);
    static_assert(CH % (kThreads / 64) == 0, "whole tiles per wavefront");
    static constexpr int kWaitVm0 = 0x0F70;  // s_waitcnt vmcnt(0), the other counters untouched
    const f32x4 *src;
    f32x4 *buf;
    int total, cur_chunk, lane, wave;

    // this wavefront's tiles [first, last) of `chunk` -> buffer b
    __device__ __forceinline__ void request(int chunk, int b, int first = 0, int last = kTilesPerWave) const {
        if (chunk >= total) chunk = total - 1;  // past the end: the last chunk again (never used)
        // (the instruction's immediate offset moves both addresses, and tiles are 1 KiB apart in memory
        // and in LDS alike: four tiles share one address computation)
        typedef __attribute__((address_space(3))) void *LdsPtr;
#pragma unroll
        for (int i = 0; i < kTilesPerWave; ++i) {
            if (i < first || i >= last) continue;
            const int tile0 = wave * kTilesPerWave + (i & ~3);
            const f32x4 *g = src + (size_t)chunk * kChunkF4 + tile0 * kTileF4 + lane;
            LdsPtr l = (LdsPtr)(buf + b * kChunkF4 + tile0 * kTileF4);
            switch (i & 3) {
                case 0: __builtin_amdgcn_global_load_lds(g, l, 16, 0, 0); break;
                case 1: __builtin_amdgcn_global_load_lds(g, l, 16, 1024, 0); break;
                case 2: __builtin_amdgcn_global_load_lds(g, l, 16, 2048, 0); break;
                default: __builtin_amdgcn_global_load_lds(g, l, 16, 3072, 0); break;
            }
        }
    }
    // Called once for every k < n by the n groups of a chunk's matrix work: the request for the
    // chunk after the current one, handed out over the first half of them (the second half of the
    // chunk is the time the last of it has to arrive).
    __device__ __forceinline__ void spread(int k, int n) const {
        const int m = n >= 2 ? n / 2 : 1;
        if (k < m) request(cur_chunk + 1, (cur_chunk + 1) & 1, k * kTilesPerWave / m, (k + 1) * kTilesPerWave / m);
    }
    __device__ __forceinline__ void start(const f32x4 *s, f32x4 *b, int n, int tid) {
        src = s; buf = b; total = n; cur_chunk = 0;
        lane = tid & 63;
        wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        request(0, 0);
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
        __syncthreads();
    }
    __device__ __forceinline__ void next() {
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
        __syncthreads();
        ++cur_chunk;
    }
    __device__ __forceinline__ f32x4 tile(int t, int lane_) const {
        return buf[(cur_chunk & 1) * kChunkF4 + t * kTileF4 + lane_];
    }
};

// VEC: N and Z are multiples of 4, so every per-lane load/store is one aligned float4 and the
// hot loops are free of branches (dead lanes and pad columns are handled by clamped addresses,
// selects and a sink buffer; control flow would force the compiler to drain all outstanding
// memory requests at every join).  DBG: per-stage outputs are stored as well.
template <int ZB, int RB, int HB, bool VEC, bool DBG>
__global__ __launch_bounds__(kThreads) void sample_chain(ChainArgs a) {
    extern __shared__ __align__(16) char lds_raw[];
    constexpr int kGuideTiles = 2 * RB * ZB + ZB * ZB;
    constexpr int Z16 = ZB * 16, R16 = RB * 16, H16 = HB * 16;
    f32x4 *gw = reinterpret_cast<f32x4 *>(lds_raw);
    f32x4 *sbuf = gw + kGuideTiles * kTileF4;
    float *ctx = reinterpret_cast<float *>(sbuf + 2 * chain_chunk_tiles(HB) * kTileF4);  // [L][R16]
    float *bias = ctx + a.L * R16;
    const int N16 = a.NB * 16;
    // bias table in LDS, in the order the layers run
    float *lb_comb = bias, *lb_mu = lb_comb + R16, *lb_sig = lb_mu + Z16;
    float *lb_gate1 = lb_sig + Z16, *lb_gate2 = lb_gate1 + H16, *lb_prop1 = lb_gate2 + Z16;
    float *lb_prop2 = lb_prop1 + H16, *lb_lin = lb_prop2 + Z16, *lb_tscale = lb_lin + Z16;
    float *lb_emean1 = lb_tscale + Z16, *lb_escale1 = lb_emean1 + H16, *lb_emean2 = lb_escale1 + H16;
    float *lb_escale2 = lb_emean2 + N16;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane >> 4;
    const int S = a.S, Z = a.Z, N = a.N;
    const int smp = (blockIdx.x * (kThreads / 64) + wave) * 16 + (lane & 15);
    const bool live = smp < S;
    const int sc = live ? smp : S - 1;  // clamped sample index for loads

    // guide weights, encodings and all biases -> LDS.  The two tables that are copied as they are go
    // straight from L2 into LDS, a 1 KiB tile per instruction (as the weight stream below); every
    // workgroup wants the same kilobytes at the same moment, so each starts at a tile of its own and
    // the requests spread over the memory channels.  Nothing waits before everything is requested.
    {
        typedef __attribute__((address_space(3))) void *LdsPtr;
        const int wv = __builtin_amdgcn_readfirstlane(wave);
        const f32x4 *src = reinterpret_cast<const f32x4 *>(a.guide_tiles);
        constexpr int kPerWave = (kGuideTiles + 3) / 4;
        const int rot = (int)(blockIdx.x % kPerWave) * 4;
#pragma unroll
        for (int j = 0; j < kPerWave; ++j) {
            int tile = j * 4 + wv + rot;
            if (tile >= kPerWave * 4) tile -= kPerWave * 4;
            if (tile < kGuideTiles)
                __builtin_amdgcn_global_load_lds(src + tile * kTileF4 + lane, (LdsPtr)(gw + tile * kTileF4), 16, 0, 0);
        }
        // all biases: one table, already in LDS order, padded to whole tiles
        const int bias_tiles = chain_bias_floats(R16, Z16, H16, N16) / 256;
        const f32x4 *bsrc = reinterpret_cast<const f32x4 *>(a.bias_table);
        for (int tile = wv; tile < bias_tiles; tile += kThreads / 64)
            __builtin_amdgcn_global_load_lds(bsrc + tile * kTileF4 + lane,
                                             (LdsPtr)(reinterpret_cast<f32x4 *>(bias) + tile * kTileF4), 16, 0, 0);
        // (1 + h_left + h_right) / 3 per position: the constant part of h_out = (tanh(.) + ...) / 3
        // with tanh written as 1 - 2 r; four positions per thread requested before the first is stored
        const int n4 = a.L * R16 / 4;
        for (int i0 = tid; i0 < n4; i0 += 4 * kThreads) {
            f32x4 f[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * kThreads < n4 ? i0 + u * kThreads : i0;
                const int t = (i * 4) / R16, r = (i * 4) % R16;
                f[u] = *reinterpret_cast<const f32x4 *>(a.ctx_f + (size_t)t * a.Rp + r);
                b[u] = *reinterpret_cast<const f32x4 *>(a.ctx_b + (size_t)t * a.Rp + r);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + u * kThreads < n4)
                    reinterpret_cast<f32x4 *>(ctx)[i0 + u * kThreads] = (f[u] + b[u] + splat(1.0f)) * (1.0f / 3.0f);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's tiles are in LDS
    }
    __syncthreads();
    auto bias4 = [&](const float *tab, int blk) { return *reinterpret_cast<const f32x4 *>(tab + blk * 16 + 4 * q); };
    const f32x4 *w_comb = gw;                         // [RB][ZB]
    const f32x4 *w_mu = gw + RB * ZB * kTileF4;       // [ZB][RB]
    const f32x4 *w_sig = gw + 2 * RB * ZB * kTileF4;  // [ZB][ZB]

    // per-lane feature mask of the latent blocks (features >= Z are padding)
    auto z_valid = [&](int zb, int v) { return zb * 16 + 4 * q + v < Z; };
    auto load_z_noise = [&](const float *base, int zb) {  // base -> [S][Z]
        f32x4 e;
        const int f0 = zb * 16 + 4 * q;
        if constexpr (VEC) {
            const int fc = f0 < Z ? f0 : Z - 4;  // clamped: always a valid address
            const f32x4 t = *reinterpret_cast<const f32x4 *>(base + (size_t)sc * Z + fc);
            const float keep = f0 < Z ? 1.f : 0.f;
            e = t * keep;
        } else {
            const float *p = base + (size_t)sc * Z + f0;
#pragma unroll
            for (int v = 0; v < 4; ++v) e[v] = z_valid(zb, v) ? p[v] : 0.f;
        }
        return e;
    };
    auto relu4 = [](f32x4 v) { return map4(v, [](float u) { return fmaxf(u, 0.f); }); };
    auto softplus4 = [](f32x4 v) { return map4(v, [](float u) { return softplus_f(u); }); };

    f32x4 z[ZB];
#pragma unroll
    for (int zb = 0; zb < ZB; ++zb) z[zb] = reinterpret_cast<const f32x4 *>(a.z0)[zb * 4 + q];

    // ---- guide chain ------------------------------------------------------------
    f32x4 eps[ZB];
#pragma unroll
    for (int zb = 0; zb < ZB; ++zb) eps[zb] = load_z_noise(a.eps_q, zb);
    for (int t = 0; t < a.L; ++t) {
        f32x4 eps_next[ZB];  // next step's noise is fetched while this step computes
        const int tn = t + 1 < a.L ? t + 1 : t;
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) eps_next[zb] = load_z_noise(a.eps_q + (size_t)tn * S * Z, zb);
        f32x4 h[RB];
        {
            // comb tiles are stored [group of GO output blocks][input block][block in group]
            constexpr int GO = RB < 4 ? RB : 4;
            const float *ctx_t = ctx + t * R16 + 4 * q;
            // h_out = (tanh(v) + h_left + h_right) / 3, tanh(v) = 1 - 2 / (exp(2v) + 1); the combiner's
            // tiles and bias carry the factor 2 log2(e) (set when the weights are loaded), so h = 2 log2(e) v
            auto finish = [&](int ob) {
                const f32x4 c = *reinterpret_cast<const f32x4 *>(ctx_t + ob * 16);  // (1 + h_left + h_right) / 3
                const f32x4 r = map4(h[ob], [](float v) { return fast_rcp(__builtin_amdgcn_exp2f(v) + 1.0f); });
                h[ob] = r * (-2.0f / 3.0f) + c;
            };
#pragma unroll
            for (int ob = 0; ob < RB; ++ob) h[ob] = bias4(lb_comb, ob);
            for_tile_groups<RB * ZB, GO>([&](int i) { return w_comb[i * kTileF4 + lane]; },
                                         [&](int g, const f32x4(&tl)[GO]) {
                                             const int og = g / ZB, ib = g % ZB;
                                             if (ib == 0 && og > 0) {  // previous group's epilogue rides along
#pragma unroll
                                                 for (int j = 0; j < GO; ++j) finish((og - 1) * GO + j);
                                             }
                                             mma_wide<GO>(&h[og * GO], tl, z[ib]);
                                         });
#pragma unroll
            for (int j = 0; j < GO; ++j) finish(RB - GO + j);
        }
        f32x4 mu[ZB];
        {
            // all ZB output blocks in one run of tiles [zb][ib]: the operand pipeline starts once
            constexpr int GI = RB < 4 ? RB : 4;
            AccN acc[ZB];
#pragma unroll
            for (int zb = 0; zb < ZB; ++zb) acc[zb].init(bias4(lb_mu, zb));
            for_tile_groups<ZB * RB, GI>([&](int i) { return w_mu[i * kTileF4 + lane]; },
                                         [&](int g, const f32x4(&tl)[GI]) {
                                             mma_narrow<GI>(acc[(g * GI) / RB], tl, &h[(g * GI) % RB]);
                                         });
#pragma unroll
            for (int zb = 0; zb < ZB; ++zb) mu[zb] = acc[zb].sum();
        }
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            AccN acc;
            acc.init(bias4(lb_sig, zb));
#pragma unroll
            for (int ib = 0; ib < ZB; ++ib) {
                const f32x4 tl[1] = {w_sig[(zb * ZB + ib) * kTileF4 + lane]};
                mma_narrow<1>(acc, tl, &mu[ib]);
            }
            z[zb] = mu[zb] + softplus4(acc.sum()) * eps[zb];
            eps[zb] = eps_next[zb];
        }
    }
    auto store_z = [&](float *dst, int ld, int zb, f32x4 v) {
        if (!DBG || !dst || !live) return;
        float *p = dst + (size_t)smp * ld + zb * 16 + 4 * q;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (z_valid(zb, k)) p[k] = v[k];
    };
#pragma unroll
    for (int zb = 0; zb < ZB; ++zb) store_z(a.z_last, Z, zb, z[zb]);

    // ---- streamed part: transition, then emission --------------------------------
    constexpr int CH = chain_chunk_tiles(HB);  // tiles per chunk
    constexpr int K2 = CH / (2 * HB);          // 16-worker blocks per chunk in the emission's output pass
    constexpr int GH = HB < 4 ? HB : 4;
    static_assert(ZB * HB <= CH && ZB * ZB <= CH, "a transition layer fits one chunk");
    WeightStream<CH> ws;
    ws.start(reinterpret_cast<const f32x4 *>(a.stream_tiles), sbuf, a.stream_chunks, tid);

    // out = W x + b for a Z -> H layer: one chunk, tiles [ib][ob]
    auto wide_from_z = [&](f32x4(&out)[HB], const float *tab, const f32x4(&x)[ZB]) {
#pragma unroll
        for (int ob = 0; ob < HB; ++ob) out[ob] = bias4(tab, ob);
        for_tile_groups<ZB * HB, GH>([&](int i) { return ws.tile(i, lane); },
                                     [&](int g, const f32x4(&tl)[GH]) {
                                         const int idx = g * GH;
                                         ws.spread(g, ZB * HB / GH);
                                         mma_wide<GH>(&out[idx % HB], tl, x[idx / HB]);
                                     });
        ws.next();
    };
    // one 16-feature output block from HB tiles starting at tile `base` of the current chunk; the
    // block is number u of the U its chunk holds (for the stream's requests)
    auto narrow_block = [&](int base, f32x4 b, const f32x4(&x)[HB], int u, int U) {
        AccN acc;
        acc.init(b);
        for_tile_groups<HB, GH>([&](int i) { return ws.tile(base + i, lane); },
                                [&](int g, const f32x4(&tl)[GH]) {
                                    ws.spread(u * (HB / GH) + g, U * (HB / GH));
                                    mma_narrow<GH>(acc, tl, &x[g * GH]);
                                });
        return acc.sum();
    };
    // out = W h + b for an H -> Z layer: one chunk, tiles [zb][ib]
    auto narrow_from_h = [&](f32x4(&out)[ZB], const float *tab, const f32x4(&x)[HB]) {
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) out[zb] = narrow_block(zb * HB, bias4(tab, zb), x, zb, ZB);
        ws.next();
    };
    // Z -> Z layer: one chunk, tiles [ob][ib]
    auto small_layer = [&](f32x4(&out)[ZB], const float *tab, const f32x4(&x)[ZB]) {
#pragma unroll
        for (int ob = 0; ob < ZB; ++ob) {
            AccN acc;
            acc.init(bias4(tab, ob));
            ws.spread(ob, ZB);
#pragma unroll
            for (int ib = 0; ib < ZB; ++ib) {
                const f32x4 tl[1] = {ws.tile(ob * ZB + ib, lane)};
                mma_narrow<1>(acc, tl, &x[ib]);
            }
            out[ob] = acc.sum();
        }
        ws.next();
    };

    f32x4 zn[ZB];
    {
        f32x4 hid[HB], g[ZB], prop[ZB], lin[ZB], G[ZB], rG[ZB], pre[ZB];
        wide_from_z(hid, lb_gate1, z);
#pragma unroll
        for (int ob = 0; ob < HB; ++ob) hid[ob] = relu4(hid[ob]);
        narrow_from_h(g, lb_gate2, hid);
        wide_from_z(hid, lb_prop1, z);
#pragma unroll
        for (int ob = 0; ob < HB; ++ob) hid[ob] = relu4(hid[ob]);
        narrow_from_h(prop, lb_prop2, hid);
        small_layer(lin, lb_lin, z);
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            const f32x4 gate = map4(g[zb], [](float v) { return sigmoid_f(v); });
            G[zb] = (splat(1.f) - gate) * lin[zb] + gate * prop[zb];
            rG[zb] = relu4(G[zb]);
        }
        small_layer(pre, lb_tscale, rG);
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            const f32x4 e = load_z_noise(a.eps_z, zb);
            zn[zb] = G[zb] + softplus4(pre[zb]) * e;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (!z_valid(zb, v)) zn[zb][v] = 0.f;
            store_z(a.z_next_dbg, Z, zb, zn[zb]);
        }
    }

    // emission: hidden layer of the mean
    f32x4 h1[HB];
    wide_from_z(h1, lb_emean1, zn);
    if (a.emit_mean_act) {
#pragma unroll
        for (int ob = 0; ob < HB; ++ob) h1[ob] = relu4(h1[ob]);
    }
    // The scale network's hidden layer.  The mean is linear in h1 and this layer is linear in the
    // mean, so it is one H x H layer on h1, M = W_J1 W_I2 and c = W_J1 b_I2 + b_J1, formed when the
    // weights are loaded (the table slot of b_J1 holds c): the N-wide mean is never an operand.
    f32x4 h2[HB];
    constexpr int RA = CH / HB;  // rows of M per chunk
#pragma unroll
    for (int c = 0; c < (HB + RA - 1) / RA; ++c) {
#pragma unroll
        for (int u = 0; u < RA; ++u) {
            const int ob = c * RA + u;
            // (rows past the end are zero tiles that fill the last chunk: only their requests are made)
            if (ob < HB) h2[ob] = relu4(narrow_block(u * HB, bias4(lb_escale1, ob), h1, u, RA));
            else ws.spread(u, RA);
        }
        ws.next();
    }

    // mean and scale of 16 workers at a time, draw, back to seconds
    const int NB = a.NB;
    const float scale = a.ctl->scale;
    float *sink = a.sink + tid * 4;
    auto load_eps_x = [&](int nb) {
        const int n0 = nb * 16 + 4 * q;
        f32x4 e = splat(0.f);
        if constexpr (VEC) {
            const int nc = n0 < N ? n0 : N - 4;
            e = *reinterpret_cast<const f32x4 *>(a.eps_x + (size_t)sc * N + nc);
        } else {
            const float *ep = a.eps_x + (size_t)sc * N + n0;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (n0 + v < N) e[v] = ep[v];
        }
        return e;
    };
    auto emit = [&](int nb, f32x4 pre, f32x4 m, f32x4 e) {  // softplus, draw, store
        const int n0 = nb * 16 + 4 * q;
        const f32x4 sd = softplus4(pre);
        const f32x4 x = (m + sd * e) * scale;
        if constexpr (VEC) {
            // columns past N and the not-yet-started pipeline slot (nb < 0) go to the sink
            float *xp = (nb >= 0 && n0 < N) ? a.out_samples + (size_t)sc * N + n0 : sink;
            *reinterpret_cast<f32x4 *>(xp) = x;
        } else {
            if (live && nb >= 0) {
                float *xp = a.out_samples + (size_t)smp * N + n0;
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (n0 + v < N) xp[v] = x[v];
            }
        }
        if constexpr (DBG) {
            if (live && nb >= 0) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if (n0 + v >= N) continue;
                    if (a.out_mean_dbg) a.out_mean_dbg[(size_t)smp * N + n0 + v] = m[v];
                    if (a.out_sd_dbg) a.out_sd_dbg[(size_t)smp * N + n0 + v] = sd[v];
                }
            }
        }
    };
    // The noise of a chunk's blocks is requested one chunk ahead, right after the weight stream's
    // own request (loads return in order: nothing waits on a request younger than one chunk).
    // Each block's epilogue rides on the next block's first matrix instructions.
    f32x4 e_next[K2];
#pragma unroll
    for (int u = 0; u < K2; ++u) e_next[u] = load_eps_x(u < NB ? u : NB - 1);
    f32x4 pre_p = splat(0.f), m_p = splat(0.f), e_p = splat(0.f);
    int nb_p = -1;  // nothing pending
    for (int c = 0; c < (NB + K2 - 1) / K2; ++c) {
        f32x4 e[K2];
#pragma unroll
        for (int u = 0; u < K2; ++u) e[u] = e_next[u];
#pragma unroll
        for (int u = 0; u < K2; ++u) {
            const int nn = (c + 1) * K2 + u;
            e_next[u] = load_eps_x(nn < NB ? nn : NB - 1);
        }
#pragma unroll
        for (int u = 0; u < K2; ++u) {
            const int nb_raw = c * K2 + u;
            const int nb = nb_raw < NB ? nb_raw : NB - 1;  // past the end: zero tiles, result goes to the sink
            // mean and scale of the block in one run of 2 HB tiles; the previous block's epilogue rides
            // on the first group
            AccN am, as;
            am.init(bias4(lb_emean2, nb));
            as.init(bias4(lb_escale2, nb));
            for_tile_groups<2 * HB, GH>([&](int i) { return ws.tile(u * 2 * HB + i, lane); },
                                        [&](int g, const f32x4(&tl)[GH]) {
                                            constexpr int kHalf = HB / GH;
                                            if (g == 0) emit(nb_p, pre_p, m_p, e_p);
                                            ws.spread(u * 2 * kHalf + g, K2 * 2 * kHalf);
                                            if (g < kHalf) mma_narrow<GH>(am, tl, &h1[g * GH]);
                                            else mma_narrow<GH>(as, tl, &h2[(g - kHalf) * GH]);
                                        });
            pre_p = as.sum(); m_p = am.sum(); e_p = e[u]; nb_p = nb_raw < NB ? nb_raw : -1;
        }
        ws.next();
    }
    emit(nb_p, pre_p, m_p, e_p);
}

template <int ZB, int RB, int HB>
size_t chain_lds_bytes(int L, int N) {
    const size_t nb16 = (size_t)((N + 15) / 16) * 16;
    const size_t bias_floats = chain_bias_floats(RB * 16, ZB * 16, HB * 16, (int)nb16);
    return (size_t)(2 * RB * ZB + ZB * ZB + 2 * chain_chunk_tiles(HB)) * kTileF4 * 16 +
           ((size_t)L * RB * 16 + bias_floats) * 4;
}

template <int ZB, int RB, int HB, bool VEC, bool DBG>
int launch_variant(const ChainArgs &a, size_t lds, hipStream_t stream) {
    static size_t raised = 0;  // largest LDS size the attribute has been set to
    if (lds > raised) {
        DKF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(sample_chain<ZB, RB, HB, VEC, DBG>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        raised = lds;
    }
    const int per_block = (kThreads / 64) * 16;
    const dim3 grid((a.S + per_block - 1) / per_block);
    hipLaunchKernelGGL((sample_chain<ZB, RB, HB, VEC, DBG>), grid, dim3(kThreads), lds, stream, a);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

template <int ZB, int RB, int HB>
int launch_one(const ChainArgs &a, hipStream_t stream) {
    const size_t lds = chain_lds_bytes<ZB, RB, HB>(a.L, a.N);
    if (lds > 160 * 1024) return DKF_EUNSUPPORTED;
    const bool vec = (a.N & 3) == 0 && (a.Z & 3) == 0 && a.N >= 4 && a.Z >= 4;
    const bool dbg = a.z_last || a.z_next_dbg || a.out_mean_dbg || a.out_sd_dbg;
    if (vec) return dbg ? launch_variant<ZB, RB, HB, true, true>(a, lds, stream)
                        : launch_variant<ZB, RB, HB, true, false>(a, lds, stream);
    return launch_variant<ZB, RB, HB, false, true>(a, lds, stream);
}

}  // namespace

bool chain_supported(int Z, int R, int H, int L, int N) {
    const int zb = (Z + 15) / 16, rb = (R + 15) / 16, hb = (H + 15) / 16;
    if (zb == 1 && rb == 2 && hb == 2) return chain_lds_bytes<1, 2, 2>(L, N) <= 160 * 1024;
    if (zb == 1 && rb == 8 && hb == 8) return chain_lds_bytes<1, 8, 8>(L, N) <= 160 * 1024;
    if (zb == 2 && rb == 16 && hb == 16) return chain_lds_bytes<2, 16, 16>(L, N) <= 160 * 1024;
    return false;
}

int launch_chain(const ChainArgs &a, hipStream_t stream) {
    StageTimer timer(kStageSampler, stream);
    const int zb = (a.Z + 15) / 16, rb = (a.R + 15) / 16, hb = (a.H + 15) / 16;
    if (zb == 1 && rb == 2 && hb == 2) return launch_one<1, 2, 2>(a, stream);
    if (zb == 1 && rb == 8 && hb == 8) return launch_one<1, 8, 8>(a, stream);
    if (zb == 2 && rb == 16 && hb == 16) return launch_one<2, 16, 16>(a, stream);
    return DKF_EUNSUPPORTED;
}

}  // namespace dkf
