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
// wavefronts of a workgroup share every fetch.  The emission scale network is
// fused back-to-back: each 16-worker block of the mean is produced, stored,
// and immediately folded into the hidden layer of the scale network.
#include "common.h"
#include "mfma_tile.h"

namespace dkf {
namespace {

constexpr int kThreads = 256;
constexpr int kTileF4 = 64;  // float4 per weight tile (one per lane)

__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// acc += W_tile (16 out x 16 in) * x (16 in x 16 samples), x held as one f32x4
__device__ __forceinline__ f32x4 tile_mma(f32x4 acc, f32x4 w, f32x4 x) {
    acc = mfma16(w.x, x.x, acc);
    acc = mfma16(w.y, x.y, acc);
    acc = mfma16(w.z, x.z, acc);
    acc = mfma16(w.w, x.w, acc);
    return acc;
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

// Double-buffered stream of weight chunks (HB tiles each) from global memory through LDS.
template <int HB>
struct WeightStream {
    static constexpr int kChunkF4 = HB * kTileF4;
    static constexpr int kPerThread = (kChunkF4 + kThreads - 1) / kThreads;
    const f32x4 *src;
    f32x4 *buf;
    int total, next_chunk, cur, tid;
    f32x4 regs[kPerThread];

    __device__ __forceinline__ void fetch(int chunk) {
        if (chunk >= total) return;
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int idx = tid + i * kThreads;
            if (idx < kChunkF4) regs[i] = src[(size_t)chunk * kChunkF4 + idx];
        }
    }
    __device__ __forceinline__ void commit(int b) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int idx = tid + i * kThreads;
            if (idx < kChunkF4) buf[b * kChunkF4 + idx] = regs[i];
        }
    }
    // chunk 0 becomes readable; chunk 1 is in flight
    __device__ __forceinline__ void start(const f32x4 *s, f32x4 *b, int n, int t) {
        src = s; buf = b; total = n; tid = t; cur = 0;
        fetch(0);
        commit(0);
        fetch(1);
        next_chunk = 2;
        __syncthreads();
    }
    // done with the current chunk: publish the next one
    __device__ __forceinline__ void advance() {
        cur ^= 1;
        commit(cur);
        fetch(next_chunk++);
        __syncthreads();
    }
    __device__ __forceinline__ f32x4 tile(int t, int lane) const { return buf[cur * kChunkF4 + t * kTileF4 + lane]; }
};

// Calls use(i, tile_i) for i = 0..COUNT-1.  Tiles are fetched GROUP at a time with the next
// group already in flight while the current one feeds the matrix cores; the scheduling fence
// after each group bounds how far ahead the compiler may hoist operand loads.
template <int COUNT, int GROUP, typename LoadF, typename UseF>
__device__ __forceinline__ void for_tiles(LoadF &&load, UseF &&use) {
    constexpr int kGroups = (COUNT + GROUP - 1) / GROUP;
    f32x4 buf[2][GROUP];
#pragma unroll
    for (int j = 0; j < GROUP; ++j)
        if (j < COUNT) buf[0][j] = load(j);
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
#pragma unroll
        for (int j = 0; j < GROUP; ++j)
            if (g + 1 < kGroups && (g + 1) * GROUP + j < COUNT) buf[(g + 1) & 1][j] = load((g + 1) * GROUP + j);
#pragma unroll
        for (int j = 0; j < GROUP; ++j)
            if (g * GROUP + j < COUNT) use(g * GROUP + j, buf[g & 1][j]);
        sched_fence();
    }
}

__device__ __forceinline__ float fast_tanh(float v) {
    // 1 - 2 / (exp(2v) + 1); exp via the hardware exp2
    const float e = __expf(2.0f * v);
    return 1.0f - __fdividef(2.0f, e + 1.0f);
}
__device__ __forceinline__ float fast_softplus(float v) {
    return fmaxf(v, 0.f) + __logf(1.0f + __expf(-fabsf(v)));
}
__device__ __forceinline__ float fast_sigmoid(float v) {
    const float e = __expf(-fabsf(v));
    const float r = __fdividef(1.0f, 1.0f + e);
    return v >= 0.f ? r : e * r;
}

template <int ZB, int RB, int HB>
__global__ __launch_bounds__(kThreads) void sample_chain(ChainArgs a) {
    extern __shared__ __align__(16) char lds_raw[];
    constexpr int kGuideTiles = 2 * RB * ZB + ZB * ZB;
    constexpr int Z16 = ZB * 16, R16 = RB * 16, H16 = HB * 16;
    constexpr int kGroup = 4;
    f32x4 *gw = reinterpret_cast<f32x4 *>(lds_raw);
    f32x4 *sbuf = gw + kGuideTiles * kTileF4;
    float *ctx = reinterpret_cast<float *>(sbuf + 2 * HB * kTileF4);  // [L][R16]
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

    // guide weights, encodings and all biases -> LDS
    {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(a.guide_tiles);
        for (int i = tid; i < kGuideTiles * kTileF4; i += kThreads) gw[i] = src[i];
        for (int i = tid; i < a.L * R16; i += kThreads) {
            const int t = i / R16, r = i % R16;
            ctx[i] = a.ctx_f[(size_t)t * a.Rp + r] + a.ctx_b[(size_t)t * a.Rp + r];
        }
        auto copy = [&](float *dst, const float *srcb, int n) {
            for (int i = tid; i < n; i += kThreads) dst[i] = srcb[i];
        };
        copy(lb_comb, a.b_comb, R16); copy(lb_mu, a.b_mu, Z16); copy(lb_sig, a.b_sig, Z16);
        copy(lb_gate1, a.b_gate1, H16); copy(lb_gate2, a.b_gate2, Z16); copy(lb_prop1, a.b_prop1, H16);
        copy(lb_prop2, a.b_prop2, Z16); copy(lb_lin, a.b_lin, Z16); copy(lb_tscale, a.b_tscale, Z16);
        copy(lb_emean1, a.b_emean1, H16); copy(lb_escale1, a.b_escale1, H16);
        copy(lb_emean2, a.b_emean2, N16); copy(lb_escale2, a.b_escale2, N16);
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
        const float *p = base + (size_t)sc * Z + zb * 16 + 4 * q;
        if ((Z & 3) == 0) {
            e = zb * 16 + 4 * q < Z ? *reinterpret_cast<const f32x4 *>(p) : splat(0.f);
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) e[v] = z_valid(zb, v) ? p[v] : 0.f;
        }
        return e;
    };
    auto relu4 = [](f32x4 v) { return map4(v, [](float u) { return fmaxf(u, 0.f); }); };
    auto softplus4 = [](f32x4 v) { return map4(v, [](float u) { return fast_softplus(u); }); };

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
            f32x4 acc;
            const float *ctx_t = ctx + t * R16 + 4 * q;
            for_tiles<RB * ZB, kGroup>(
                [&](int i) { return w_comb[i * kTileF4 + lane]; },
                [&](int i, f32x4 w) {
                    const int ob = i / ZB, ib = i % ZB;
                    if (ib == 0) acc = bias4(lb_comb, ob);
                    acc = tile_mma(acc, w, z[ib]);
                    if (ib == ZB - 1) {
                        const f32x4 c = *reinterpret_cast<const f32x4 *>(ctx_t + ob * 16);
                        h[ob] = (map4(acc, [](float v) { return fast_tanh(v); }) + c) * (1.0f / 3.0f);
                    }
                });
        }
        f32x4 mu[ZB];
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            f32x4 acc0 = bias4(lb_mu, zb), acc1 = splat(0.f);
            for_tiles<RB, kGroup>([&](int i) { return w_mu[(zb * RB + i) * kTileF4 + lane]; },
                                  [&](int i, f32x4 w) {
                                      if (i & 1) acc1 = tile_mma(acc1, w, h[i]);
                                      else acc0 = tile_mma(acc0, w, h[i]);
                                  });
            mu[zb] = acc0 + acc1;
        }
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            f32x4 acc = bias4(lb_sig, zb);
#pragma unroll
            for (int ib = 0; ib < ZB; ++ib) acc = tile_mma(acc, w_sig[(zb * ZB + ib) * kTileF4 + lane], mu[ib]);
            z[zb] = mu[zb] + softplus4(acc) * eps[zb];
            eps[zb] = eps_next[zb];
        }
    }
    auto store_z = [&](float *dst, int ld, int zb, f32x4 v) {
        if (!dst || !live) return;
        float *p = dst + (size_t)smp * ld + zb * 16 + 4 * q;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (z_valid(zb, k)) p[k] = v[k];
    };
#pragma unroll
    for (int zb = 0; zb < ZB; ++zb) store_z(a.z_last, Z, zb, z[zb]);

    // ---- streamed part: transition, then emission --------------------------------
    WeightStream<HB> ws;
    ws.start(reinterpret_cast<const f32x4 *>(a.stream_tiles), sbuf, a.stream_chunks, tid);
    constexpr int kSmall = (ZB * ZB + HB - 1) / HB;  // chunks holding a Z x Z layer

    // out = W1 x + b1 for a Z -> H layer streamed as ZB chunks (one per input block)
    auto wide_from_z = [&](f32x4(&out)[HB], const float *tab, const f32x4(&x)[ZB]) {
#pragma unroll
        for (int ob = 0; ob < HB; ++ob) out[ob] = bias4(tab, ob);
#pragma unroll
        for (int ib = 0; ib < ZB; ++ib) {
            for_tiles<HB, kGroup>([&](int i) { return ws.tile(i, lane); },
                                  [&](int i, f32x4 w) { out[i] = tile_mma(out[i], w, x[ib]); });
            ws.advance();
        }
    };
    // one 16-feature output block of an H -> . layer streamed as one chunk
    auto narrow_from_h = [&](f32x4 b, const f32x4(&x)[HB]) {
        f32x4 acc0 = b, acc1 = splat(0.f);
        for_tiles<HB, kGroup>([&](int i) { return ws.tile(i, lane); },
                              [&](int i, f32x4 w) {
                                  if (i & 1) acc1 = tile_mma(acc1, w, x[i]);
                                  else acc0 = tile_mma(acc0, w, x[i]);
                              });
        ws.advance();
        return acc0 + acc1;
    };
    // Z -> Z layer, tiles [ob][ib] packed into kSmall chunks
    auto small_layer = [&](f32x4(&out)[ZB], const float *tab, const f32x4(&x)[ZB]) {
#pragma unroll
        for (int ob = 0; ob < ZB; ++ob) out[ob] = bias4(tab, ob);
#pragma unroll
        for (int c = 0; c < kSmall; ++c) {
#pragma unroll
            for (int i = 0; i < HB; ++i) {
                const int idx = c * HB + i;
                if (idx < ZB * ZB) out[idx / ZB] = tile_mma(out[idx / ZB], ws.tile(i, lane), x[idx % ZB]);
            }
            ws.advance();
        }
    };

    f32x4 zn[ZB];
    {
        f32x4 hid[HB], g[ZB], prop[ZB], lin[ZB], G[ZB], rG[ZB], pre[ZB];
        wide_from_z(hid, lb_gate1, z);
#pragma unroll
        for (int ob = 0; ob < HB; ++ob) hid[ob] = relu4(hid[ob]);
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb)
            g[zb] = map4(narrow_from_h(bias4(lb_gate2, zb), hid), [](float v) { return fast_sigmoid(v); });
        wide_from_z(hid, lb_prop1, z);
#pragma unroll
        for (int ob = 0; ob < HB; ++ob) hid[ob] = relu4(hid[ob]);
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) prop[zb] = narrow_from_h(bias4(lb_prop2, zb), hid);
        small_layer(lin, lb_lin, z);
#pragma unroll
        for (int zb = 0; zb < ZB; ++zb) {
            G[zb] = (splat(1.f) - g[zb]) * lin[zb] + g[zb] * prop[zb];
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

    // emission
    f32x4 h1[HB];
    wide_from_z(h1, lb_emean1, zn);
    if (a.emit_mean_act) {
#pragma unroll
        for (int ob = 0; ob < HB; ++ob) h1[ob] = relu4(h1[ob]);
    }
    f32x4 h2[HB];
#pragma unroll
    for (int ob = 0; ob < HB; ++ob) h2[ob] = bias4(lb_escale1, ob);
    const int NB = a.NB;
    float *mean_row = a.mean + (size_t)sc * a.ld_mean + 4 * q;
    for (int nb = 0; nb < NB; ++nb) {
        const f32x4 m = narrow_from_h(bias4(lb_emean2, nb), h1);
        if (live) *reinterpret_cast<f32x4 *>(mean_row + nb * 16) = m;
        for_tiles<HB, kGroup>([&](int i) { return ws.tile(i, lane); },
                              [&](int i, f32x4 w) { h2[i] = tile_mma(h2[i], w, m); });
        ws.advance();
    }
#pragma unroll
    for (int ob = 0; ob < HB; ++ob) h2[ob] = relu4(h2[ob]);
    const float scale = a.ctl->scale;
    const bool vec_ok = (N & 3) == 0;
    for (int nb = 0; nb < NB; ++nb) {
        const int n0 = nb * 16 + 4 * q;
        const f32x4 m = *reinterpret_cast<const f32x4 *>(mean_row + nb * 16);
        f32x4 e = splat(0.f);
        const float *ep = a.eps_x + (size_t)sc * N + n0;
        if (vec_ok) {
            if (n0 < N) e = *reinterpret_cast<const f32x4 *>(ep);
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (n0 + v < N) e[v] = ep[v];
        }
        const f32x4 sd = softplus4(narrow_from_h(bias4(lb_escale2, nb), h2));
        const f32x4 x = (m + sd * e) * scale;
        if (live) {
            float *xp = a.out_samples + (size_t)smp * N + n0;
            if (vec_ok) {
                if (n0 < N) *reinterpret_cast<f32x4 *>(xp) = x;
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (n0 + v < N) xp[v] = x[v];
            }
            if (a.out_mean_dbg || a.out_sd_dbg) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if (n0 + v >= N) continue;
                    if (a.out_mean_dbg) a.out_mean_dbg[(size_t)smp * N + n0 + v] = m[v];
                    if (a.out_sd_dbg) a.out_sd_dbg[(size_t)smp * N + n0 + v] = sd[v];
                }
            }
        }
    }
}

template <int ZB, int RB, int HB>
size_t chain_lds_bytes(int L, int N) {
    const size_t nb16 = (size_t)((N + 15) / 16) * 16;
    const size_t bias_floats = RB * 16 + 6 * ZB * 16 + 4 * HB * 16 + 2 * nb16;
    return (size_t)(2 * RB * ZB + ZB * ZB + 2 * HB) * kTileF4 * 16 + ((size_t)L * RB * 16 + bias_floats) * 4;
}

template <int ZB, int RB, int HB>
int launch_one(const ChainArgs &a, hipStream_t stream) {
    const size_t lds = chain_lds_bytes<ZB, RB, HB>(a.L, a.N);
    if (lds > 160 * 1024) return DKF_EUNSUPPORTED;
    static size_t raised = 0;  // largest LDS size the attribute has been set to
    if (lds > raised) {
        DKF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(sample_chain<ZB, RB, HB>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        raised = lds;
    }
    const int per_block = (kThreads / 64) * 16;
    const dim3 grid((a.S + per_block - 1) / per_block);
    hipLaunchKernelGGL((sample_chain<ZB, RB, HB>), grid, dim3(kThreads), lds, stream, a);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
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
    StageTimer timer(kStageGuide, stream);
    const int zb = (a.Z + 15) / 16, rb = (a.R + 15) / 16, hb = (a.H + 15) / 16;
    if (zb == 1 && rb == 2 && hb == 2) return launch_one<1, 2, 2>(a, stream);
    if (zb == 1 && rb == 8 && hb == 8) return launch_one<1, 8, 8>(a, stream);
    if (zb == 2 && rb == 16 && hb == 16) return launch_one<2, 16, 16>(a, stream);
    return DKF_EUNSUPPORTED;
}

}  // namespace dkf
