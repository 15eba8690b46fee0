// Posterior-predictive sampling for a few thousand samples (Sec. 3.1.3): the chain of layers of
// chain.hip -- L guide steps, the gated transition draw, the emission draw -- with sixteen samples
// per WORKGROUP instead of per wavefront.  The W (four or eight) wavefronts of a workgroup work on
// the same sixteen samples and split every layer between them, so that 4096 samples put one or two
// wavefronts on every SIMD of the chip while each matrix instruction still carries sixteen samples.
// Two per SIMD is what pays: a wavefront's vector work does not run in the shadow of its own matrix
// instructions, another wavefront's does.
//
// How a layer is split (activation blocks of 16 features x 16 samples as in mfma16.h):
//   wide layers   (Z -> R, Z -> H):  by output blocks; every wavefront holds the whole latent, so
//                                    nothing is exchanged before the layer;
//   narrow layers (R -> Z, H -> Z):  by input blocks, each wavefront using the share of the hidden
//                                    features it has just computed itself; the W partial results
//                                    are added through LDS in a fixed order ((w0 + w1) + w2) + ...,
//                                    after which every wavefront holds the whole latent again;
//   Z -> Z layers:                   computed by all wavefronts alike;
//   emission:  the mean's hidden layer is computed by output blocks and gathered through LDS.  The
//              scale network's first layer is linear in the mean and the mean linear in that
//              hidden layer, so it is applied as their H x H product (formed when the weights are
//              loaded): a second hidden layer, again by output blocks and gathered.  Both stay in
//              LDS (an operand block is read per tile).  After that a wavefront owns a contiguous
//              share of the workers and, for each of its 16-worker blocks, forms mean and scale
//              from the two hidden layers and draws.
// One exchange per guide step, one for the transition, two for the emission.
//
// Weights: a wavefront only ever touches its own share of every matrix.  Its share of the guide's
// three matrices stays in registers for the L steps; everything else is laid out, when the
// weights are loaded (pack_split, api.hip), as one stream per wavefront in exactly the order it is
// consumed, and flows from L2 straight into a ring of registers one block of work ahead of the
// matrix instructions: no staging in LDS, no barrier for the weights.
#include "common.h"
#include "mfma_tile.h"
#include "mfma16.h"
#include "rowsort.h"
#include <type_traits>

namespace dkf {
namespace {

constexpr int kTileF4 = 64;

template <int ZB, int RB, int HB, int W>
struct SplitShape {
    static_assert(RB % 4 == 0 && HB % W == 0, "hidden widths split four and W ways");
    static constexpr int GW = 4;                               // wavefronts that run the guide chain
    static constexpr int RQ = RB / GW, HQ = HB / W;
    static constexpr int kGuide = 2 * RQ * ZB + ZB * ZB;       // tiles held in registers (wavefronts below GW)
    // ring size: the tiles of one emission block (mean row + scale row), or half of that where two
    // wavefronts share a SIMD's registers
    static constexpr int C = W == 8 ? HB : 2 * HB;
    static constexpr int kBlockChunks = 2 * HB / C;
    static constexpr int kHead = 5 * HQ * ZB + 2 * ZB * ZB;    // gate1 gate2 prop1 prop2 lin tscale emean1
    static constexpr int kHeadChunks = (kHead + C - 1) / C;
    static constexpr int kFold = HQ * HB;                      // this wavefront's rows of the folded layer
    static constexpr int kFoldChunks = (kFold + C - 1) / C;
    // tiles of one wavefront's stream for nbw worker blocks per wavefront (one spare chunk at the end:
    // the ring always requests one chunk ahead)
    __host__ __device__ static constexpr int stream_tiles(int nbw) {
        return kGuide + (kHeadChunks + kFoldChunks + nbw * kBlockChunks + 1) * C;
    }
};

// SLG > 0: the workgroup also sorts its sixteen rows (N = 8 << SLG workers) and writes their rank sums.
template <int ZB, int RB, int HB, int W, bool DBG, int SLG = 0>
__global__ __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(W / 4, W / 4))) void sample_split(ChainArgs a) {
    using Sh = SplitShape<ZB, RB, HB, W>;
    constexpr int RQ = Sh::RQ, HQ = Sh::HQ, C = Sh::C, kThreads = 64 * W;
    constexpr int Z16 = ZB * 16, R16 = RB * 16, H16 = HB * 16;
    extern __shared__ __align__(16) char lds_raw[];
    // LDS: exchange buffers, then the encodings' table and the bias table
    f32x4 *x_mu = reinterpret_cast<f32x4 *>(lds_raw);          // [2][W][2 ZB][64]  latent-sized partial sums
    f32x4 *x_h1 = x_mu + 2 * W * 2 * ZB * kTileF4;             // [HB][64]          hidden layer of the mean
    f32x4 *x_h2 = x_h1 + HB * kTileF4;                         // [HB][64]          hidden layer of the scale
    f32x4 *x_sum = x_h2 + HB * kTileF4;                        // [ZB][64]          the latent after the guide chain (W = 8)
    float *ctx = reinterpret_cast<float *>(x_sum + ZB * kTileF4);  // [L][R16]
    float *bias = ctx + a.L * R16;
    const int NB = a.NB, N16 = NB * 16;
    const int NBW = (NB + W - 1) / W;  // worker blocks per wavefront
    float *lb_comb = bias, *lb_mu = lb_comb + R16, *lb_sig = lb_mu + Z16;
    float *lb_gate1 = lb_sig + Z16, *lb_gate2 = lb_gate1 + H16, *lb_prop1 = lb_gate2 + Z16;
    float *lb_prop2 = lb_prop1 + H16, *lb_lin = lb_prop2 + Z16, *lb_tscale = lb_lin + Z16;
    float *lb_emean1 = lb_tscale + Z16, *lb_escale1 = lb_emean1 + H16, *lb_emean2 = lb_escale1 + H16;
    float *lb_escale2 = lb_emean2 + N16;

    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane >> 4;
    const int S = a.S, Z = a.Z, N = a.N;
    const int smp = blockIdx.x * 16 + (lane & 15);
    const bool live = smp < S;
    const int sc = live ? smp : S - 1;  // clamped sample index: lanes past the end repeat the last sample

    // this wavefront's weight stream
    const f32x4 *T = reinterpret_cast<const f32x4 *>(a.stream_tiles) + (size_t)w * Sh::stream_tiles(NBW) * kTileF4 + lane;
    f32x4 wc[RQ][ZB], wm[ZB][RQ], wsg[ZB][ZB];
    if (w < Sh::GW) {
#pragma unroll
        for (int o = 0; o < RQ; ++o)
#pragma unroll
            for (int ib = 0; ib < ZB; ++ib) wc[o][ib] = T[(o * ZB + ib) * kTileF4];
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb)
#pragma unroll
            for (int i = 0; i < RQ; ++i) wm[zb][i] = T[(RQ * ZB + zb * RQ + i) * kTileF4];
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb)
#pragma unroll
            for (int ib = 0; ib < ZB; ++ib) wsg[zb][ib] = T[(2 * RQ * ZB + zb * ZB + ib) * kTileF4];
    }
    // ring of the streamed tiles: slot i holds tile i of the current chunk; taking it requests tile i
    // of the next chunk into the same slot
    const f32x4 *cur = T + (size_t)Sh::kGuide * kTileF4;
    f32x4 ring[C];
#pragma unroll
    for (int i = 0; i < C; ++i) ring[i] = cur[i * kTileF4];
    auto take = [&](int i) {
        const f32x4 t = ring[i];
        ring[i] = cur[(C + i) * kTileF4];
        return t;
    };

    // encodings and biases -> LDS
    {
        // (1 + h_left + h_right) / 3 per position: the constant part of h_out = (tanh(.) + ...) / 3
        // with tanh written as 1 - 2 r
        const int n4 = a.L * R16 / 4;
        for (int i = tid; i < n4; i += kThreads) {
            const int t = (i * 4) / R16, r = (i * 4) % R16;
            const f32x4 f = *reinterpret_cast<const f32x4 *>(a.ctx_f + (size_t)t * a.Rp + r);
            const f32x4 b = *reinterpret_cast<const f32x4 *>(a.ctx_b + (size_t)t * a.Rp + r);
            reinterpret_cast<f32x4 *>(ctx)[i] = (f + b + splat(1.0f)) * (1.0f / 3.0f);
        }
        const int b4 = (R16 + 6 * Z16 + 4 * H16 + 2 * N16) / 4;
        const f32x4 *bsrc = reinterpret_cast<const f32x4 *>(a.bias_table);
        for (int i = tid; i < b4; i += kThreads) reinterpret_cast<f32x4 *>(bias)[i] = bsrc[i];
    }
    __syncthreads();
    auto bias4 = [&](const float *tab, int blk) { return *reinterpret_cast<const f32x4 *>(tab + blk * 16 + 4 * q); };
    auto z_valid = [&](int zb, int v) { return zb * 16 + 4 * q + v < Z; };
    auto load_z_noise = [&](const float *base, int zb) {  // base -> [S][Z]; Z is a multiple of 4
        const int f0 = zb * 16 + 4 * q;
        const int fc = f0 < Z ? f0 : Z - 4;  // clamped: always a valid address
        const f32x4 t = *reinterpret_cast<const f32x4 *>(base + (size_t)sc * Z + fc);
        return t * (f0 < Z ? 1.f : 0.f);
    };
    auto relu4 = [](f32x4 v) { return map4(v, [](float u) { return fmaxf(u, 0.f); }); };
    auto softplus4 = [](f32x4 v) { return map4(v, [](float u) { return softplus_f(u); }); };

    // Sum of the partial blocks p[0..n) of wavefronts 0 .. G-1, in the order ((w0 + w1) + w2) + ...;
    // each of them ends up with the same full result.  Every wavefront of the workgroup must make
    // the call (it holds a barrier); two buffers alternate, so one barrier per call.
    int xbuf = 0;
    auto all_sum = [&](auto &p, auto group) {
        constexpr int n = sizeof(p) / sizeof(p[0]), G = decltype(group)::value;
        static_assert(n <= 2 * ZB && G <= W, "exchange buffer size");
        if (w < G) {
            f32x4 *mine = x_mu + ((xbuf * W + w) * 2 * ZB) * kTileF4 + lane;
#pragma unroll
            for (int i = 0; i < n; ++i) mine[i * kTileF4] = p[i];
        }
        __syncthreads();
        if (w < G) {
            const f32x4 *all = x_mu + (xbuf * W * 2 * ZB) * kTileF4 + lane;
#pragma unroll
            for (int i = 0; i < n; ++i) {
                const f32x4 *e = all + i * kTileF4;
                f32x4 sum = e[0];
#pragma unroll
                for (int k = 1; k < G; ++k) sum = sum + e[k * 2 * ZB * kTileF4];
                p[i] = sum;
            }
        }
        xbuf ^= 1;
    };
    constexpr std::integral_constant<int, Sh::GW> kGuideGroup{};
    constexpr std::integral_constant<int, W> kEveryone{};

    f32x4 z[ZB];
#pragma unroll
    for (int zb = 0; zb < ZB; ++zb) z[zb] = reinterpret_cast<const f32x4 *>(a.z0)[zb * 4 + q];

    // ---- guide chain ------------------------------------------------------------------
    // The chain is one dependent sequence of small layers with an exchange per step: more than four
    // wavefronts only make the exchange dearer (measured), so with eight the upper four sit out the
    // chain at its barriers and receive the latent at the end.
    f32x4 eps[ZB];
#pragma unroll
    for (int zb = 0; zb < ZB; ++zb) eps[zb] = w < Sh::GW ? load_z_noise(a.eps_q, zb) : splat(0.f);
    for (int t = 0; t < a.L; ++t) {
        if (w >= Sh::GW) {  // (uniform per wavefront)
            f32x4 none[ZB];
            all_sum(none, kGuideGroup);
            continue;
        }
        f32x4 eps_next[ZB];  // next step's noise is fetched while this step computes
        const int tn = t + 1 < a.L ? t + 1 : t;
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) eps_next[zb] = load_z_noise(a.eps_q + (size_t)tn * S * Z, zb);
        // this wavefront's quarter of h_out = (tanh(W z + b) + h_left + h_right) / 3
        f32x4 h[RQ];
#pragma unroll
        for (int o = 0; o < RQ; ++o) h[o] = bias4(lb_comb, w * RQ + o);
#pragma unroll
        for (int ib = 0; ib < ZB; ++ib) {
            f32x4 tl[RQ];
#pragma unroll
            for (int o = 0; o < RQ; ++o) tl[o] = wc[o][ib];
            mma_wide<RQ>(h, tl, z[ib]);
        }
        const float *ctx_t = ctx + t * R16 + 4 * q;
#pragma unroll
        for (int o = 0; o < RQ; ++o) {
            const f32x4 c = *reinterpret_cast<const f32x4 *>(ctx_t + (w * RQ + o) * 16);  // (1 + h_left + h_right) / 3
            const f32x4 r = map4(h[o], [](float v) { return fast_rcp(__expf(2.0f * v) + 1.0f); });
            h[o] = r * (-2.0f / 3.0f) + c;
        }
        // mean: partial product over this wavefront's hidden features, then the sum over wavefronts
        f32x4 mu[ZB];
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            Acc4 acc;
            acc.init(splat(0.f));
            f32x4 tl[RQ];
#pragma unroll
            for (int i = 0; i < RQ; ++i) tl[i] = wm[zb][i];
            mma_narrow<RQ>(acc, tl, h);
            mu[zb] = acc.sum();
        }
        all_sum(mu, kGuideGroup);
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) mu[zb] = mu[zb] + bias4(lb_mu, zb);
        // scale from the mean, reparameterised draw (all wavefronts alike)
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            Acc4 acc;
            acc.init(bias4(lb_sig, zb));
#pragma unroll
            for (int ib = 0; ib < ZB; ++ib) {
                const f32x4 tl[1] = {wsg[zb][ib]};
                mma_narrow<1>(acc, tl, &mu[ib]);
            }
            z[zb] = mu[zb] + softplus4(acc.sum()) * eps[zb];
            eps[zb] = eps_next[zb];
        }
    }
    auto store_z = [&](float *dst, int zb, f32x4 v) {
        if (!DBG || !dst || !live || w != 0) return;
        float *p = dst + (size_t)smp * Z + zb * 16 + 4 * q;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (z_valid(zb, k)) p[k] = v[k];
    };
#pragma unroll
    for (int zb = 0; zb < ZB; ++zb) store_z(a.z_last, zb, z[zb]);
    if constexpr (W > Sh::GW) {  // the latent for the wavefronts that sat out
        if (w == 0) {
#pragma unroll
            for (int zb = 0; zb < ZB; ++zb) x_sum[zb * kTileF4 + lane] = z[zb];
        }
        __syncthreads();
        if (w >= Sh::GW) {
#pragma unroll
            for (int zb = 0; zb < ZB; ++zb) z[zb] = x_sum[zb * kTileF4 + lane];
        }
    }

    // ---- gated transition -----------------------------------------------------------------
    // ring positions of the head of the stream (compile-time): gate1, gate2, prop1, prop2, lin, tscale, emean1
    constexpr int pG1 = 0, pG2 = pG1 + HQ * ZB, pP1 = pG2 + ZB * HQ, pP2 = pP1 + HQ * ZB, pLin = pP2 + ZB * HQ,
                  pTs = pLin + ZB * ZB, pE1 = pTs + ZB * ZB;
    static_assert(pE1 + HQ * ZB == Sh::kHead, "head layout");
    // The head may span several chunks of the ring; `head_take` follows a compile-time position.
    int head_chunk = 0;
    auto head_take = [&](int pos) {  // positions are visited in increasing order
        if (pos / C != head_chunk) { cur += C * kTileF4; head_chunk = pos / C; }
        return take(pos % C);
    };
    // this wavefront's quarter of a Z -> H layer
    auto wide_quarter = [&](f32x4(&out)[HQ], const float *tab, int pos, const f32x4(&x)[ZB]) {
        f32x4 tl[ZB][HQ];  // stream order [o][ib]; all tiles first, so that the HQ accumulator chains can advance in turn
#pragma unroll
        for (int o = 0; o < HQ; ++o)
#pragma unroll
            for (int ib = 0; ib < ZB; ++ib) tl[ib][o] = head_take(pos + o * ZB + ib);
#pragma unroll
        for (int o = 0; o < HQ; ++o) out[o] = bias4(tab, w * HQ + o);
#pragma unroll
        for (int ib = 0; ib < ZB; ++ib) mma_wide<HQ>(out, tl[ib], x[ib]);
    };
    // partial product of an H -> Z layer over this wavefront's quarter of the hidden features (no bias)
    auto narrow_quarter = [&](f32x4(&out)[ZB], int pos, const f32x4(&x)[HQ]) {
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            Acc4 acc;
            acc.init(splat(0.f));
#pragma unroll
            for (int i = 0; i < HQ; ++i) {  // stream order [zb][i]
                const f32x4 tl[1] = {head_take(pos + zb * HQ + i)};
                mma_narrow<1>(acc, tl, &x[i]);
            }
            out[zb] = acc.sum();
        }
    };
    auto small_layer = [&](f32x4(&out)[ZB], const float *tab, int pos, const f32x4(&x)[ZB]) {
#pragma unroll
        for (int ob = 0; ob < ZB; ++ob) {
            Acc4 acc;
            acc.init(bias4(tab, ob));
#pragma unroll
            for (int ib = 0; ib < ZB; ++ib) {
                const f32x4 tl[1] = {head_take(pos + ob * ZB + ib)};
                mma_narrow<1>(acc, tl, &x[ib]);
            }
            out[ob] = acc.sum();
        }
    };

    f32x4 zn[ZB];
    {
        f32x4 hid[HQ], g[ZB], prop[ZB], gp[2 * ZB], lin[ZB], G[ZB], rG[ZB], pre[ZB];
        wide_quarter(hid, lb_gate1, pG1, z);
#pragma unroll
        for (int o = 0; o < HQ; ++o) hid[o] = relu4(hid[o]);
        narrow_quarter(g, pG2, hid);
        wide_quarter(hid, lb_prop1, pP1, z);
#pragma unroll
        for (int o = 0; o < HQ; ++o) hid[o] = relu4(hid[o]);
        narrow_quarter(prop, pP2, hid);
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) { gp[zb] = g[zb]; gp[ZB + zb] = prop[zb]; }
        all_sum(gp, kEveryone);  // gate and proposed mean in one exchange
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) { g[zb] = gp[zb]; prop[zb] = gp[ZB + zb]; }
        small_layer(lin, lb_lin, pLin, z);
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            const f32x4 gate = map4(g[zb] + bias4(lb_gate2, zb), [](float v) { return sigmoid_f(v); });
            G[zb] = (splat(1.f) - gate) * lin[zb] + gate * (prop[zb] + bias4(lb_prop2, zb));
            rG[zb] = relu4(G[zb]);
        }
        small_layer(pre, lb_tscale, pTs, rG);
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            const f32x4 e = load_z_noise(a.eps_z, zb);
            zn[zb] = G[zb] + softplus4(pre[zb]) * e;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (!z_valid(zb, v)) zn[zb][v] = 0.f;
            store_z(a.z_next_dbg, zb, zn[zb]);
        }
    }

    // ---- emission ---------------------------------------------------------------------------
    // noise of this wavefront's worker blocks, requested now
    const float scale = a.ctl->scale;
    float *sink = a.sink + tid * 4;
    const int nb0 = w * NBW;  // first of this wavefront's worker blocks
    auto load_eps_x = [&](int nb) {
        const int n0 = nb * 16 + 4 * q;
        const int nc = n0 < N ? n0 : N - 4;
        return *reinterpret_cast<const f32x4 *>(a.eps_x + (size_t)sc * N + nc);
    };
    // hidden layer of the mean: own share of the output blocks, gathered in LDS
    {
        f32x4 own[HQ];
        wide_quarter(own, lb_emean1, pE1, zn);
        if (a.emit_mean_act) {
#pragma unroll
            for (int o = 0; o < HQ; ++o) own[o] = relu4(own[o]);
        }
#pragma unroll
        for (int o = 0; o < HQ; ++o) x_h1[(w * HQ + o) * kTileF4 + lane] = own[o];
        __syncthreads();
    }
    // the rest of the head's last chunk is padding: taking it lets the ring request the next chunk's tiles
#pragma unroll
    for (int pos = Sh::kHead; pos < Sh::kHeadChunks * C; ++pos) (void)head_take(pos);
    cur += C * kTileF4;  // the ring now holds the first chunk of the folded layer
    // hidden layer of the scale network from the mean's (the folded H x H layer; the table slot of
    // b_J1 holds its bias): own share of the output blocks, row by row, gathered in LDS
    {
        f32x4 own[HQ];
#pragma unroll
        for (int o = 0; o < HQ; ++o) {
            Acc4 acc;
            acc.init(bias4(lb_escale1, w * HQ + o));
#pragma unroll
            for (int i = 0; i < HB; ++i) {
                const f32x4 tl[1] = {take((o * HB + i) % C)};
                const f32x4 x = x_h1[i * kTileF4 + lane];
                mma_narrow<1>(acc, tl, &x);
                if ((o * HB + i + 1) % C == 0) cur += C * kTileF4;
                if (i % 4 == 3) sched_fence();  // bounds how many operand blocks are fetched ahead
            }
            own[o] = relu4(acc.sum());
        }
        if constexpr (Sh::kFold % C != 0) {  // padding of the last chunk
#pragma unroll
            for (int i = Sh::kFold % C; i < C; ++i) (void)take(i);
            cur += C * kTileF4;
        }
#pragma unroll
        for (int o = 0; o < HQ; ++o) x_h2[(w * HQ + o) * kTileF4 + lane] = own[o];
        __syncthreads();
    }
    // rows of the workgroup for the sort below: [16][N + 4] floats (the pad keeps the sixteen samples
    // of a store on different banks), then the wavefronts' rank sums [W][8][N / 8]
    constexpr int kSortStride = (8 << SLG) + 4;
    float *sort_rows = reinterpret_cast<float *>(x_mu);
    static_assert(SLG == 0 || (16 * kSortStride + W * (8 << SLG)) * 4 <= 2 * W * 2 * ZB * kTileF4 * 16, "sort buffers fit the exchange buffers");
    // mean, scale, draw, back to seconds: per worker block HB tiles of the mean's output layer, row nb,
    // then HB tiles of the scale's (one chunk of the ring, or two)
    auto emit = [&](int nb_raw, f32x4 pre, f32x4 m, f32x4 e) {
        const int n0 = nb_raw * 16 + 4 * q;
        const f32x4 sd = softplus4(pre);
        const f32x4 x = (m + sd * e) * scale;
        // lanes past the last sample repeat sample S - 1 exactly (a harmless duplicate store); columns
        // past N and blocks past the end go to the sink
        float *xp = (nb_raw < NB && n0 < N) ? a.out_samples + (size_t)sc * N + n0 : sink;
        *reinterpret_cast<f32x4 *>(xp) = x;
        if constexpr (SLG > 0) {  // and into this workgroup's copy of its sixteen rows (exchange buffers: free by now)
            if (nb_raw < NB) *reinterpret_cast<f32x4 *>(sort_rows + (lane & 15) * kSortStride + n0) = x;
        }
        if constexpr (DBG) {
            if (live && nb_raw < NB) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if (n0 + v >= N) continue;
                    if (a.out_mean_dbg) a.out_mean_dbg[(size_t)smp * N + n0 + v] = m[v];
                    if (a.out_sd_dbg) a.out_sd_dbg[(size_t)smp * N + n0 + v] = sd[v];
                }
            }
        }
    };
    f32x4 e_next = load_eps_x(nb0 < NB ? nb0 : NB - 1);  // noise one block ahead
    for (int u = 0; u < NBW; ++u) {
        const int nb_raw = nb0 + u, nb = nb_raw < NB ? nb_raw : NB - 1;  // past the end: zero tiles, result to the sink
        const f32x4 e = e_next;
        e_next = load_eps_x(nb_raw + 1 < NB ? nb_raw + 1 : NB - 1);
        Acc4 am, as;
        am.init(bias4(lb_emean2, nb));
        as.init(bias4(lb_escale2, nb));
        if constexpr (Sh::kBlockChunks == 1) {
#pragma unroll
            for (int i = 0; i < HB; ++i) {
                const f32x4 tm[1] = {take(i)}, ts[1] = {take(HB + i)};
                const f32x4 x1 = x_h1[i * kTileF4 + lane], x2 = x_h2[i * kTileF4 + lane];
                mma_narrow<1>(am, tm, &x1);
                mma_narrow<1>(as, ts, &x2);
                if (i % 4 == 3) sched_fence();
            }
            cur += C * kTileF4;
        } else {
#pragma unroll
            for (int i = 0; i < HB; ++i) {
                const f32x4 tm[1] = {take(i)};
                const f32x4 x1 = x_h1[i * kTileF4 + lane];
                mma_narrow<1>(am, tm, &x1);
                if (i % 4 == 3) sched_fence();
            }
            cur += C * kTileF4;
#pragma unroll
            for (int i = 0; i < HB; ++i) {
                const f32x4 ts[1] = {take(i)};
                const f32x4 x2 = x_h2[i * kTileF4 + lane];
                mma_narrow<1>(as, ts, &x2);
                if (i % 4 == 3) sched_fence();
            }
            cur += C * kTileF4;
        }
        emit(nb_raw, as.sum(), am.sum(), e);
    }
    // ---- order statistics of the sixteen rows (Sec. 3.1.1, last paragraph) -------------------
    // A lane group of N / 8 lanes sorts one row, eight keys per lane, exactly as the row-sort
    // kernel does; the rank sums of the workgroup's rows are added in a fixed order and written as
    // row blockIdx.x of the table rank_means_omega reduces.
    if constexpr (SLG > 0) {
        constexpr int E = 8, G = 1 << SLG, NPAD = E * G, RPW = 64 / G;  // RPW rows per wavefront at a time
        static_assert(16 % RPW == 0, "whole passes");
        using Lay = Layout<E, SLG>;
        float *red = sort_rows + 16 * kSortStride;  // [W][E][G]
        __syncthreads();  // every wavefront's worker blocks of the sixteen rows have been written
        const int g = lane & (G - 1), sub = lane >> SLG;
        float acc[E];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = 0.f;
        for (int r0 = w * RPW; r0 < 16; r0 += W * RPW) {  // (the same trips for every lane of a wavefront)
            const float *src = sort_rows + (r0 + sub) * kSortStride;
            uint32_t v[E];
#pragma unroll
            for (int qq = 0; qq < E / 4; ++qq) {
                const f32x4 t = *reinterpret_cast<const f32x4 *>(src + Lay::load_index(g, qq * 4));
                v[qq * 4] = key_of_flat(t[0]); v[qq * 4 + 1] = key_of_flat(t[1]);
                v[qq * 4 + 2] = key_of_flat(t[2]); v[qq * 4 + 3] = key_of_flat(t[3]);
            }
            sort_in_lane<uint32_t, E>(v);
            merge_up<uint32_t, E, SLG, Lay::kLgE + 1>(v, g);
#pragma unroll
            for (int e = 0; e < E; ++e) acc[e] += value_of(v[e]);
        }
#pragma unroll
        for (int d = G; d < 64; d <<= 1) {
#pragma unroll
            for (int e = 0; e < E; ++e) acc[e] += __shfl_xor(acc[e], d, 64);
        }
        if (lane < G) {
#pragma unroll
            for (int e = 0; e < E; ++e) red[(w * E + e) * G + lane] = acc[e];
        }
        __syncthreads();
        for (int idx = tid; idx < E * G; idx += kThreads) {
            const int e = idx / G, gg = idx % G;
            float sum = red[e * G + gg];
#pragma unroll
            for (int k = 1; k < W; ++k) sum += red[(k * E + e) * G + gg];
            a.rank_partial[(size_t)blockIdx.x * NPAD + Lay::rank(gg, e)] = sum;
        }
        if (blockIdx.x == 0 && tid == 0) *a.rank_done = 0u;  // the counter of the reduction that follows
    }
}

template <int ZB, int RB, int HB, int W>
size_t split_lds_bytes(int L, int N) {
    const size_t nb16 = (size_t)((N + 15) / 16) * 16;
    const size_t bias_floats = RB * 16 + 6 * ZB * 16 + 4 * HB * 16 + 2 * nb16;
    return (size_t)(2 * W * 2 * ZB + HB + HB + ZB) * kTileF4 * 16 + ((size_t)L * RB * 16 + bias_floats) * 4;
}

template <int ZB, int RB, int HB, int W, bool DBG, int SLG = 0>
int launch_variant(const ChainArgs &a, size_t lds, hipStream_t stream) {
    static size_t raised = 0;  // largest LDS size the attribute has been set to
    if (lds > raised) {
        DKF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(sample_split<ZB, RB, HB, W, DBG, SLG>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        raised = lds;
    }
    hipLaunchKernelGGL((sample_split<ZB, RB, HB, W, DBG, SLG>), dim3((a.S + 15) / 16), dim3(64 * W), lds, stream, a);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

template <int ZB, int RB, int HB, int W>
int launch_one(const ChainArgs &a, hipStream_t stream) {
    const size_t lds = split_lds_bytes<ZB, RB, HB, W>(a.L, a.N);
    if (lds > 160 * 1024) return DKF_EUNSUPPORTED;
    const bool dbg = a.z_last || a.z_next_dbg || a.out_mean_dbg || a.out_sd_dbg;
    if (a.rank_partial) {  // the caller has asked split_sorts_rows
        if constexpr (W == 8) {
            if (dbg || !a.rank_done || a.S % 16 != 0) return DKF_EINVAL;
            if (a.N == 128) return launch_variant<ZB, RB, HB, W, false, 4>(a, lds, stream);
            if constexpr (ZB >= 2) {  // (the rows of 512 workers need the exchange buffers of the wider latent)
                if (a.N == 512) return launch_variant<ZB, RB, HB, W, false, 6>(a, lds, stream);
            }
        }
        return DKF_EUNSUPPORTED;
    }
    return dbg ? launch_variant<ZB, RB, HB, W, true>(a, lds, stream) : launch_variant<ZB, RB, HB, W, false>(a, lds, stream);
}

}  // namespace

// Sizes the kernel is built for: the latent and the widths of the two larger fp32 presets, N and Z
// multiples of 4, and as many workers as leave the bias table room in LDS.  waves: wavefronts per
// workgroup, 4 or 8.
bool split_supported(int Z, int R, int H, int L, int N, int waves) {
    const int zb = (Z + 15) / 16, rb = (R + 15) / 16, hb = (H + 15) / 16;
    if (N < 4 || (N & 3) != 0 || Z < 4 || (Z & 3) != 0 || (waves != 4 && waves != 8)) return false;
    if (zb == 1 && rb == 8 && hb == 8)
        return (waves == 4 ? split_lds_bytes<1, 8, 8, 4>(L, N) : split_lds_bytes<1, 8, 8, 8>(L, N)) <= 160 * 1024;
    if (zb == 2 && rb == 16 && hb == 16)
        return (waves == 4 ? split_lds_bytes<2, 16, 16, 4>(L, N) : split_lds_bytes<2, 16, 16, 8>(L, N)) <= 160 * 1024;
    return false;
}

bool split_sorts_rows(int Z, int R, int H, int L, int N, int S, int waves) {
    const int zb = (Z + 15) / 16;
    return waves == 8 && (N == 128 || (N == 512 && zb >= 2)) && S >= 16 && S % 16 == 0 &&
           split_supported(Z, R, H, L, N, waves);
}

int split_stream_tiles(int Z, int R, int H, int N, int waves) {
    const int zb = (Z + 15) / 16, rb = (R + 15) / 16, hb = (H + 15) / 16, nbw = ((N + 15) / 16 + waves - 1) / waves;
    if (zb == 1 && rb == 8 && hb == 8)
        return waves == 4 ? SplitShape<1, 8, 8, 4>::stream_tiles(nbw) : SplitShape<1, 8, 8, 8>::stream_tiles(nbw);
    if (zb == 2 && rb == 16 && hb == 16)
        return waves == 4 ? SplitShape<2, 16, 16, 4>::stream_tiles(nbw) : SplitShape<2, 16, 16, 8>::stream_tiles(nbw);
    return 0;
}

int launch_split(const ChainArgs &a, hipStream_t stream) {
    StageTimer timer(kStageSampler, stream);
    const int zb = (a.Z + 15) / 16, rb = (a.R + 15) / 16, hb = (a.H + 15) / 16;
    if (!split_supported(a.Z, a.R, a.H, a.L, a.N, a.split_waves)) return DKF_EUNSUPPORTED;
    if (zb == 1 && rb == 8 && hb == 8)
        return a.split_waves == 4 ? launch_one<1, 8, 8, 4>(a, stream) : launch_one<1, 8, 8, 8>(a, stream);
    if (zb == 2 && rb == 16 && hb == 16)
        return a.split_waves == 4 ? launch_one<2, 16, 16, 4>(a, stream) : launch_one<2, 16, 16, 8>(a, stream);
    return DKF_EUNSUPPORTED;
}

}  // namespace dkf
