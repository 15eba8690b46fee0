// Guide trajectories and the gated transition in bf16 (Sec. 3.1.3) with the
// guide's weights held in registers for all L steps.
//
// A workgroup of four wavefronts (one per SIMD) owns 32 samples.  Every layer
// is computed transposed, Y^T = W X^T, with v_mfma_f32_32x32x16_bf16: weights
// are the A operand (rows = output features), activations the B operand
// (columns = samples).  Lane l of a result tile owns sample l % 32 and features
// 8 (i / 4) + 4 (l / 32) + i % 4, i = 0..15; with the weights' K order permuted
// the same way at load time, a result tile rounded to bf16 *is* two B operands
// of the next layer, so activations never leave registers inside a wavefront.
//   wide layers  (Z -> R, Z -> H): each wavefront computes a quarter of the
//                output features from the full latent (which every wavefront holds);
//   narrow layers (R -> Z, H -> Z): each wavefront multiplies its quarter of the
//                hidden features (K split) and the four partial results are summed
//                through LDS in a fixed order;
//   in the guide's steps the latent is then finished by quarters: wavefront w
//                owns the eight registers per lane that make up B fragment w of the
//                latent, sums, scales (Z -> Z product for its tile), draws and rounds
//                only those, and the four fragments are handed round through LDS;
//   the transition ends the same way (gate, linear branch, scale and draw by quarters), and
//                the hidden layer of the emission's mean follows while z_{T+1} is at hand.
// The context enters the mean linearly, mu = W_mu (tanh(.) + h_l + h_r) / 3 + b,
// so its share c_t = W_mu (h_l,t + h_r,t) / 3 + b_mu is computed once per window
// position by guide_context (fp32, unrounded weights) and added after the
// matrix product: the per-sample work of a step is tanh on the accumulators and
// three products.  Transition weights are used once per workgroup and are
// fetched from L2, all at once, in the same tile format.
#include "common.h"
#include "mfma_tile.h"

namespace dkf {
namespace {

constexpr int kThreads = 256;
constexpr int kRows = 32;  // samples per workgroup
constexpr int ZT = 2;      // 32-feature tiles of the latent (Zp = 64)
constexpr int ZK = 4;      // 16-wide k-steps of the latent

__device__ __forceinline__ f32x16 mma(bf16x8 w, bf16x8 x, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, x, c, 0, 0, 0);
}

// half G (0/1) of a result tile as the B operand of k-step 2 * tile + G of the next layer
template <int G>
__device__ __forceinline__ bf16x8 operand_of(const f32x16 &v) {
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = (__bf16)v[8 * G + j];  // round to nearest even
    return r;
}

__device__ __forceinline__ bf16x8 load_tile(const f32x4 *__restrict__ tiles, int tile, int lane) {
    return __builtin_bit_cast(bf16x8, tiles[(size_t)tile * 64 + lane]);
}

// c_t[z] = b_mu[z] + (1/3) sum_r W_mu[z][r] (ctx_f[t][r] + ctx_b[t][r]);  grid (L, ceil(Z/4)), one wavefront per z
__global__ __launch_bounds__(256) void guide_context(GChainArgs a) {
    if (a.ctl->count < a.L) return;
    const int t = blockIdx.x, z = blockIdx.y * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (z >= a.Z) return;
    const float *__restrict__ w = a.mu_w32 + (size_t)z * a.R;
    const float *__restrict__ cf = a.ctx_f + (size_t)t * a.Rp;
    const float *__restrict__ cb = a.ctx_b + (size_t)t * a.Rp;
    float s = 0.f;
    for (int r = lane; r < a.R; r += 64) s += w[r] * (cf[r] + cb[r]);
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) s += __shfl_xor(s, d, 64);
    if (lane == 0) a.cmu[(size_t)t * 64 + z] = s * (1.0f / 3.0f) + a.mu_b32[z];
}

// Q: 32-feature tiles of the hidden width per wavefront (hidden widths padded to 128 Q).
template <int Q>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void guide_chain_bf16(GChainArgs a) {
    extern __shared__ __align__(16) char lds_raw[];
    // LDS: red[2][4][8][64] float4 (two exchange buffers for partial sums), frags[3][4][64] float4
    // (hand-over of finished quarters), bias table, c_t table
    f32x4 *red = reinterpret_cast<f32x4 *>(lds_raw);
    f32x4 *frags = red + 2 * 4 * 8 * 64;  // [3][4][64]: quarters of a latent-sized vector as bf16 B fragments
    float *bias = reinterpret_cast<float *>(frags + 3 * 4 * 64);
    float *cmu = bias + a.bias_floats;
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int col = lane & 31, h = lane >> 5;
    const int S = a.S, Z = a.Z, L = a.L;
    const int smp = blockIdx.x * kRows + col;
    const bool live = smp < S;
    const f32x4 *__restrict__ T = reinterpret_cast<const f32x4 *>(a.tiles);
    constexpr int HP = 128 * Q;  // padded hidden width
    // bias table offsets (floats)
    constexpr int oC = 0, oSig = oC + HP, oG1 = oSig + 64, oG2 = oG1 + HP, oP1 = oG2 + 64, oP2 = oP1 + HP,
                  oLin = oP2 + 64, oTs = oLin + 64, oE1 = oTs + 64;
    // tile offsets
    constexpr int nWide = 4 * Q * ZK, nNarrow = 4 * ZT * 2 * Q, nSmall = ZT * ZK;
    constexpr int tC = 0, tMu = tC + nWide, tSig = tMu + nNarrow, tG1 = tSig + nSmall, tG2 = tG1 + nWide,
                  tP1 = tG2 + nNarrow, tP2 = tP1 + nWide, tLin = tP2 + nNarrow, tTs = tLin + nSmall, tE1 = tTs + nSmall;

    // tables -> LDS, eight loads in flight per thread (a load-store loop would pay one memory round
    // trip per iteration)
    auto stage_table = [&](float *dst, const float *__restrict__ src, int n) {
        for (int i0 = tid; i0 < n; i0 += 8 * kThreads) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = i0 + u * kThreads < n ? src[i0 + u * kThreads] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (i0 + u * kThreads < n) dst[i0 + u * kThreads] = v[u];
        }
    };
    stage_table(bias, a.bias_table, a.bias_floats);
    stage_table(cmu, a.cmu, L * 64);

    // guide weights of this wavefront -> registers
    bf16x8 wc[Q][ZK], wmu[ZT][2 * Q], wsig[ZK];  // of the scale's matrix only the tile of this wavefront's quarter
#pragma unroll
    for (int ob = 0; ob < Q; ++ob)
#pragma unroll
        for (int ks = 0; ks < ZK; ++ks) wc[ob][ks] = load_tile(T, tC + (w * Q + ob) * ZK + ks, lane);
#pragma unroll
    for (int nb = 0; nb < ZT; ++nb)
#pragma unroll
        for (int ks = 0; ks < 2 * Q; ++ks) wmu[nb][ks] = load_tile(T, tMu + (w * ZT + nb) * 2 * Q + ks, lane);
#pragma unroll
    for (int ks = 0; ks < ZK; ++ks) wsig[ks] = load_tile(T, tSig + (w >> 1) * ZK + ks, lane);

    // z_0 as B operands: k-step ks, entry j <-> feature 16 ks + 8 (j / 4) + 4 h + j % 4
    bf16x8 zB[ZK];
#pragma unroll
    for (int ks = 0; ks < ZK; ++ks)
#pragma unroll
        for (int j = 0; j < 8; ++j) zB[ks][j] = (__bf16)a.z0[16 * ks + 8 * (j >> 2) + 4 * h + (j & 3)];
    __syncthreads();

    // accumulator tile that starts at the bias of this lane's 16 features (read from the LDS table)
    auto bias_tile = [&](const float *b) {  // b: table entry of the tile's first feature + 4 h
        f32x16 v;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 bq = *reinterpret_cast<const f32x4 *>(b + 8 * q);
            v[4 * q] = bq[0]; v[4 * q + 1] = bq[1]; v[4 * q + 2] = bq[2]; v[4 * q + 3] = bq[3];
        }
        return v;
    };

    // After the combiner and the mean's partial products a step continues on QUARTERS of the latent:
    // wavefront w owns the eight registers per lane that are B fragment w of the latent (tile
    // w / 2, registers 8 (w % 2) ..).  It adds the four partial sums of its quarter, finishes the mean
    // there, hands the quarter to the others as one bf16 fragment, multiplies the scale's product
    // for its tile from the four fragments, applies softplus and draws on its quarter only, and
    // hands the new latent over the same way.  (Every wavefront finishing the whole latent by itself
    // costs four times the transcendental work of this part and four times the LDS reads.)
    // Three barriers per step; each buffer is written two barriers after its last read.
    const int own_tile = w >> 1, own_half = w & 1;
    f32x4 *frag_mu = frags, *frag_z = frags + 4 * 64, *frag_g = frags + 8 * 64;
    float zq[8] = {};  // this wavefront's quarter of z_t, fp32
    // this quarter's features: register j <-> 32 own_tile + 16 own_half + 8 (j / 4) + 4 h + j % 4
    const int qfeat0 = 32 * own_tile + 16 * own_half + 4 * h;
    for (int t = 0; t < L; ++t) {
        f32x4 eps[2];
        {
            const float *__restrict__ row = a.eps_q + ((size_t)t * S + (live ? smp : 0)) * Z;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int f = qfeat0 + 8 * q;
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
                if (live && f < Z) v = *reinterpret_cast<const f32x4 *>(row + f);
                eps[q] = v;
            }
        }
        // combiner: this wavefront's quarter of W_c z + b_c, all products issued before the first tanh
        // (k-step outermost: consecutive matrix instructions then belong to different accumulators;
        // one that continues the accumulator of the instruction just before it waits out its latency)
        f32x16 pre[Q];
#pragma unroll
        for (int ob = 0; ob < Q; ++ob) pre[ob] = bias_tile(bias + oC + 32 * (w * Q + ob) + 4 * h);
#pragma unroll
        for (int ks = 0; ks < ZK; ++ks)
#pragma unroll
            for (int ob = 0; ob < Q; ++ob) pre[ob] = mma(wc[ob][ks], zB[ks], pre[ob]);
        // tanh tile by tile, each straight into two B operands of the mean's partial product over
        // this wavefront's hidden features
        f32x16 mu[ZT];
#pragma unroll
        for (int nb = 0; nb < ZT; ++nb) mu[nb] = zero16();
#pragma unroll
        for (int ob = 0; ob < Q; ++ob) {
#pragma unroll
            for (int i = 0; i < 16; ++i) pre[ob][i] = tanh_f(pre[ob][i]);
            const bf16x8 h0 = operand_of<0>(pre[ob]), h1 = operand_of<1>(pre[ob]);
#pragma unroll
            for (int nb = 0; nb < ZT; ++nb) mu[nb] = mma(wmu[nb][2 * ob], h0, mu[nb]);
#pragma unroll
            for (int nb = 0; nb < ZT; ++nb) mu[nb] = mma(wmu[nb][2 * ob + 1], h1, mu[nb]);
        }
        // partial sums -> LDS; own quarter summed in the order ((w0 + w1) + w2) + w3
        {
            f32x4 *mine = red + (w * 8) * 64 + lane;
#pragma unroll
            for (int nb = 0; nb < ZT; ++nb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 v = {mu[nb][4 * q], mu[nb][4 * q + 1], mu[nb][4 * q + 2], mu[nb][4 * q + 3]};
                    mine[(nb * 4 + q) * 64] = v;
                }
        }
        __syncthreads();
        float muq[8];
        {
            const f32x4 *all = red + lane;
            const float *c = cmu + t * 64 + qfeat0;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int e = (own_tile * 4 + 2 * own_half + q) * 64;
                const f32x4 s4 = ((all[e] + all[8 * 64 + e]) + all[16 * 64 + e]) + all[24 * 64 + e];
                const f32x4 cq = *reinterpret_cast<const f32x4 *>(c + 8 * q);
#pragma unroll
                for (int r = 0; r < 4; ++r) muq[4 * q + r] = s4[r] * (1.0f / 3.0f) + cq[r];
            }
        }
        {
            bf16x8 mq;
#pragma unroll
            for (int j = 0; j < 8; ++j) mq[j] = (__bf16)muq[j];
            frag_mu[w * 64 + lane] = __builtin_bit_cast(f32x4, mq);
        }
        __syncthreads();
        // scale from the mean (this wavefront's tile only), reparameterised draw on its quarter.  Pad
        // features need no masking: their mean is 0 (zero weight rows, zero c_t) and their noise was
        // loaded as 0.
        f32x16 sg = bias_tile(bias + oSig + 32 * own_tile + 4 * h);
#pragma unroll
        for (int ks = 0; ks < ZK; ++ks) sg = mma(wsig[ks], __builtin_bit_cast(bf16x8, frag_mu[ks * 64 + lane]), sg);
        {
            // (two copies of the loop, each with constant register numbers: one loop that picks its
            // half at run time is compiled into a sixteen-way select per element)
            bf16x8 zb8;
            if (own_half) {
#pragma unroll
                for (int j = 0; j < 8; ++j) zq[j] = muq[j] + softplus_f(sg[8 + j]) * eps[j >> 2][j & 3];
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) zq[j] = muq[j] + softplus_f(sg[j]) * eps[j >> 2][j & 3];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) zb8[j] = (__bf16)zq[j];
            frag_z[w * 64 + lane] = __builtin_bit_cast(f32x4, zb8);
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < ZK; ++ks) zB[ks] = __builtin_bit_cast(bf16x8, frag_z[ks * 64 + lane]);
    }
    if (a.z_last && live) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int f = qfeat0 + 8 * q;
            if (f < Z) {
                f32x4 v = {zq[4 * q], zq[4 * q + 1], zq[4 * q + 2], zq[4 * q + 3]};
                *reinterpret_cast<f32x4 *>(a.z_last + (size_t)smp * Z + f) = v;
            }
        }
    }

    // ---- gated transition and the emission's first layer: weights used once per workgroup.  All of
    // them are requested here, at once, into the registers the guide's weights occupied: one L2 round
    // trip for the whole tail instead of one per layer. ---------------------------------------------
    bf16x8 wg1[Q][ZK], wg2[ZT][2 * Q], wp1[Q][ZK], wp2[ZT][2 * Q], wl[ZK], wt[ZK], we[Q][ZK];
#pragma unroll
    for (int ob = 0; ob < Q; ++ob)
#pragma unroll
        for (int ks = 0; ks < ZK; ++ks) {
            wg1[ob][ks] = load_tile(T, tG1 + (w * Q + ob) * ZK + ks, lane);
            wp1[ob][ks] = load_tile(T, tP1 + (w * Q + ob) * ZK + ks, lane);
            we[ob][ks] = load_tile(T, tE1 + (w * Q + ob) * ZK + ks, lane);
        }
#pragma unroll
    for (int nb = 0; nb < ZT; ++nb)
#pragma unroll
        for (int ks = 0; ks < 2 * Q; ++ks) {
            wg2[nb][ks] = load_tile(T, tG2 + (w * ZT + nb) * 2 * Q + ks, lane);
            wp2[nb][ks] = load_tile(T, tP2 + (w * ZT + nb) * 2 * Q + ks, lane);
        }
#pragma unroll
    for (int ks = 0; ks < ZK; ++ks) {  // of the two Z -> Z layers only the tile of this wavefront's quarter
        wl[ks] = load_tile(T, tLin + own_tile * ZK + ks, lane);
        wt[ks] = load_tile(T, tTs + own_tile * ZK + ks, lane);
    }
    f32x4 epz[2];
    {
        const float *__restrict__ row = a.eps_z + (size_t)(live ? smp : 0) * Z;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int f = qfeat0 + 8 * q;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (live && f < Z) v = *reinterpret_cast<const f32x4 *>(row + f);
            epz[q] = v;
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // wide layer (Z -> H) of this wavefront's quarter + ReLU, then the narrow layer's partial
    // product over that quarter; the partial sums go to exchange buffer `xb`
    auto two_layer = [&](const bf16x8 (&ww)[Q][ZK], int o_wide, const bf16x8 (&wn)[ZT][2 * Q], int xb) {
        f32x16 pre[Q], out[ZT];
#pragma unroll
        for (int ob = 0; ob < Q; ++ob) pre[ob] = bias_tile(bias + o_wide + 32 * (w * Q + ob) + 4 * h);
#pragma unroll
        for (int ks = 0; ks < ZK; ++ks)
#pragma unroll
            for (int ob = 0; ob < Q; ++ob) pre[ob] = mma(ww[ob][ks], zB[ks], pre[ob]);
#pragma unroll
        for (int nb = 0; nb < ZT; ++nb) out[nb] = zero16();
#pragma unroll
        for (int ob = 0; ob < Q; ++ob) {
#pragma unroll
            for (int i = 0; i < 16; ++i) pre[ob][i] = fmaxf(pre[ob][i], 0.f);
            const bf16x8 h0 = operand_of<0>(pre[ob]), h1 = operand_of<1>(pre[ob]);
#pragma unroll
            for (int nb = 0; nb < ZT; ++nb) out[nb] = mma(wn[nb][2 * ob], h0, out[nb]);
#pragma unroll
            for (int nb = 0; nb < ZT; ++nb) out[nb] = mma(wn[nb][2 * ob + 1], h1, out[nb]);
        }
        f32x4 *mine = red + ((xb * 4 + w) * 8) * 64 + lane;
#pragma unroll
        for (int nb = 0; nb < ZT; ++nb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f32x4 v = {out[nb][4 * q], out[nb][4 * q + 1], out[nb][4 * q + 2], out[nb][4 * q + 3]};
                mine[(nb * 4 + q) * 64] = v;
            }
    };
    // this wavefront's quarter of the sum of the four partial tiles in buffer xb, ((w0 + w1) + w2) + w3
    auto quarter_sum = [&](int xb, float (&s8)[8]) {
        const f32x4 *all = red + (xb * 4 * 8) * 64 + lane;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int e = (own_tile * 4 + 2 * own_half + q) * 64;
            const f32x4 s4 = ((all[e] + all[8 * 64 + e]) + all[16 * 64 + e]) + all[24 * 64 + e];
#pragma unroll
            for (int r = 0; r < 4; ++r) s8[4 * q + r] = s4[r];
        }
    };
    // own half (eight registers) of a result tile, with constant register numbers in either case
    auto own_regs = [&](const f32x16 &t, float (&o8)[8]) {
        if (own_half) {
#pragma unroll
            for (int j = 0; j < 8; ++j) o8[j] = t[8 + j];
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) o8[j] = t[j];
        }
    };
    two_layer(wg1, oG1, wg2, 0);
    two_layer(wp1, oP1, wp2, 1);
    // the Z -> Z layer of the linear branch, for the tile of this wavefront's quarter
    f32x16 lin = bias_tile(bias + oLin + 32 * own_tile + 4 * h);
#pragma unroll
    for (int ks = 0; ks < ZK; ++ks) lin = mma(wl[ks], zB[ks], lin);
    __syncthreads();
    float gq[8], pq[8], lq[8], Gq[8];
    quarter_sum(0, gq);
    quarter_sum(1, pq);
    own_regs(lin, lq);
    {
        bf16x8 g8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int f = qfeat0 + 8 * (j >> 2) + (j & 3);
            const float g = sigmoid_f(gq[j] + bias[oG2 + f]);
            const float v = (1.f - g) * lq[j] + g * (pq[j] + bias[oP2 + f]);
            Gq[j] = f < Z ? v : 0.f;
            g8[j] = (__bf16)fmaxf(Gq[j], 0.f);
        }
        frag_g[w * 64 + lane] = __builtin_bit_cast(f32x4, g8);
    }
    __syncthreads();
    f32x16 ts = bias_tile(bias + oTs + 32 * own_tile + 4 * h);
#pragma unroll
    for (int ks = 0; ks < ZK; ++ks) ts = mma(wt[ks], __builtin_bit_cast(bf16x8, frag_g[ks * 64 + lane]), ts);
    float tq[8], znq[8];
    own_regs(ts, tq);
    {
        bf16x8 z8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int f = qfeat0 + 8 * (j >> 2) + (j & 3);
            const float zn = Gq[j] + softplus_f(tq[j]) * epz[j >> 2][j & 3];
            znq[j] = f < Z ? zn : 0.f;
            z8[j] = (__bf16)znq[j];
        }
        // (rows beyond S too: finite padding for the layers that follow)
        frag_z[w * 64 + lane] = __builtin_bit_cast(f32x4, z8);
    }
    if (live) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int f = qfeat0 + 8 * q;
            const f32x4 v = {znq[4 * q], znq[4 * q + 1], znq[4 * q + 2], znq[4 * q + 3]};
            if (a.z_next) *reinterpret_cast<f32x4 *>(a.z_next + (size_t)smp * a.Zp + f) = v;
            if (a.z_next_dbg && f < Z) *reinterpret_cast<f32x4 *>(a.z_next_dbg + (size_t)smp * Z + f) = v;
        }
    }
    // Hidden layer of the emission's mean (Z -> H), while z_{T+1} is at hand: each wavefront multiplies
    // its quarter of the output features and writes them as the B fragments the emission's kernels read.
    if (a.h1frag) {
        __syncthreads();
        bf16x8 znB[ZK];
#pragma unroll
        for (int ks = 0; ks < ZK; ++ks) znB[ks] = __builtin_bit_cast(bf16x8, frag_z[ks * 64 + lane]);
        f32x16 pre[Q];
#pragma unroll
        for (int ob = 0; ob < Q; ++ob) pre[ob] = bias_tile(bias + oE1 + 32 * (w * Q + ob) + 4 * h);
#pragma unroll
        for (int ks = 0; ks < ZK; ++ks)
#pragma unroll
            for (int ob = 0; ob < Q; ++ob) pre[ob] = mma(we[ob][ks], znB[ks], pre[ob]);
#pragma unroll
        for (int ob = 0; ob < Q; ++ob) {
            const int mb = w * Q + ob;
            if (2 * mb >= a.h1_k_steps) continue;  // feature blocks past the emission's padded width
            if (a.emit_mean_act) {
#pragma unroll
                for (int i = 0; i < 16; ++i) pre[ob][i] = fmaxf(pre[ob][i], 0.f);
            }
            f32x4 *out = reinterpret_cast<f32x4 *>(a.h1frag) + ((size_t)blockIdx.x * a.h1_k_steps + 2 * mb) * 64 + lane;
            out[0] = __builtin_bit_cast(f32x4, operand_of<0>(pre[ob]));
            out[64] = __builtin_bit_cast(f32x4, operand_of<1>(pre[ob]));
        }
    }
}

size_t gchain_lds(const GChainArgs &a) {
    return (size_t)(2 * 4 * 8 + 3 * 4) * 64 * 16 + ((size_t)a.bias_floats + (size_t)a.L * 64) * sizeof(float);
}

template <int Q>
int launch_q(const GChainArgs &a, hipStream_t stream) {
    const size_t lds = gchain_lds(a);
    if (lds > 160 * 1024) return DKF_EUNSUPPORTED;
    static size_t prepared = 0;  // largest LDS size the kernel has been enabled for
    if (lds > prepared) {
        DKF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(guide_chain_bf16<Q>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        prepared = lds;
    }
    hipLaunchKernelGGL(guide_context, dim3(a.L, (a.Z + 3) / 4), dim3(256), 0, stream, a);
    DKF_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(guide_chain_bf16<Q>, dim3((a.S + kRows - 1) / kRows), dim3(kThreads), lds, stream, a);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

}  // namespace

int gchain_q(int Z, int R, int H) {
    if (Z < 1 || Z > 64 || (Z & 3) != 0) return 0;
    const int widest = R > H ? R : H;
    if (widest <= 128) return 1;
    if (widest <= 256) return 2;
    if (widest <= 512) return 4;
    return 0;
}

int launch_gchain(const GChainArgs &a, hipStream_t stream) {
    StageTimer timer(kStageGuide, stream);
    if ((reinterpret_cast<uintptr_t>(a.eps_q) | reinterpret_cast<uintptr_t>(a.eps_z) |
         reinterpret_cast<uintptr_t>(a.z_last) | reinterpret_cast<uintptr_t>(a.z_next_dbg)) & 15)
        return DKF_EINVAL;
    switch (gchain_q(a.Z, a.R, a.H)) {
        case 1: return launch_q<1>(a, stream);
        case 2: return launch_q<2>(a, stream);
        case 4: return launch_q<4>(a, stream);
        default: return DKF_EUNSUPPORTED;
    }
}

}  // namespace dkf
