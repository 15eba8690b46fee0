// Guide trajectories and the gated transition for a tile of 32 samples per
// workgroup (Sec. 3.1.3):
//   for t = 1..L:  h_out = (tanh(W_c z + b_c) + h_left,t + h_right,t) / 3
//                  mu = W_mu h_out + b_mu;  sigma = softplus(W_sig mu + b_sig)
//                  z = mu + sigma * eps_q[t]
//   g = sigmoid(W_g2 relu(W_g1 z + b) + b);  h = W_h2 relu(W_h1 z + b) + b
//   G = (1 - g) (W_l z + b_l) + g h;  Hs = softplus(W_s relu(G) + b_s)
//   z' = G + Hs * eps_z
// The chain is sequential in t but independent across samples, so one kernel
// keeps a sample tile's state in LDS for all L steps and the transition; every
// layer is a 32-row MFMA product against weights streamed from L2.
// Wide layers (Z -> R, Z -> H) give each wavefront its own 32-column blocks;
// narrow ones (R -> Z, H -> Z) split the K range over the four wavefronts and
// add the partial tiles in a fixed order.
#include "common.h"
#include "mfma_tile.h"

namespace dkf {
namespace {

constexpr int kThreads = 256;
constexpr int kRows = 32;        // samples per workgroup
constexpr int kLda = kRows + 1;  // plane stride of an A tile, in 16-byte entries

struct Lds {
    f32x4 *zA;    // [Zp/PL][kLda]  current latent, as an A operand (PL = columns per plane)
    f32x4 *hA;    // [max(Rp,Hp)/PL][kLda]  h_out, then the hidden layers of the transition
    f32x4 *mA;    // [Zp/PL][kLda]  mu, later relu(G)
    float *red;   // [4][1024] partial accumulator tiles
    float *gT;    // [32][Zp] gate
    float *linT;  // [32][Zp] linear branch
    float *GT;    // [32][Zp] fp32 mu during the guide steps, then the transition mean
};

template <bool BF16>
__device__ __forceinline__ Lds carve(char *base, int Zp, int Wp) {
    constexpr int PL = BF16 ? 8 : 4;
    Lds l;
    size_t off = 0;
    l.zA = reinterpret_cast<f32x4 *>(base + off); off += (size_t)(Zp / PL) * kLda * 16;
    l.hA = reinterpret_cast<f32x4 *>(base + off); off += (size_t)(Wp / PL) * kLda * 16;
    l.mA = reinterpret_cast<f32x4 *>(base + off); off += (size_t)(Zp / PL) * kLda * 16;
    l.red = reinterpret_cast<float *>(base + off); off += 4 * 1024 * 4;
    l.gT = reinterpret_cast<float *>(base + off); off += (size_t)kRows * Zp * 4;
    l.linT = reinterpret_cast<float *>(base + off); off += (size_t)kRows * Zp * 4;
    l.GT = reinterpret_cast<float *>(base + off);
    return l;
}

__device__ __forceinline__ const f32x4 *block_tiles(const PackedLayer &p, int nb) {
    return reinterpret_cast<const f32x4 *>(p.tiles) + (size_t)nb * p.k_groups * 64;
}

// Wide layer: out[32][n_blocks*32] = f(A * W + b), one 32-column block per wavefront pass.
template <bool BF16, typename F>
__device__ __forceinline__ void wide_layer(const PackedLayer &p, const f32x4 *A, int wave, int lane, F &&store) {
    for (int nb = wave; nb < p.n_blocks; nb += kThreads / 64) {
        f32x16 acc = zero16();
        mma_block<BF16>(acc, A, kLda, 0, block_tiles(p, nb), 0, p.k_groups, lane);
        const int col = nb * 32 + (lane & 31);
        const float b = p.bias[col];
#pragma unroll
        for (int i = 0; i < 16; ++i) store(acc_row(i, lane), col, acc[i] + b);
    }
}

// Narrow layer: K split over the four wavefronts, partial tiles summed as
// ((w0 + w1) + w2) + w3.  `store(row, col, value_with_bias)` runs once per element.
template <bool BF16, typename F>
__device__ __forceinline__ void narrow_layer(const PackedLayer &p, const f32x4 *A, float *red, int wave, int lane,
                                             F &&store) {
    const int tid = wave * 64 + lane;
    const int per = (p.k_groups + 3) / 4;
    for (int nb = 0; nb < p.n_blocks; ++nb) {
        f32x16 acc = zero16();
        const int kg0 = wave * per;
        const int kg1 = min(kg0 + per, p.k_groups);
        if (kg0 < kg1) mma_block<BF16>(acc, A, kLda, 0, block_tiles(p, nb), kg0, kg1, lane);
#pragma unroll
        for (int i = 0; i < 16; ++i) red[wave * 1024 + i * 64 + lane] = acc[i];
        __syncthreads();
        for (int idx = tid; idx < 1024; idx += kThreads) {
            const float s = ((red[idx] + red[1024 + idx]) + red[2048 + idx]) + red[3072 + idx];
            const int i = idx >> 6, l = idx & 63;
            const int col = nb * 32 + (l & 31);
            store(acc_row(i, l), col, s + p.bias[col]);
        }
        __syncthreads();
    }
}

// BF16: every matrix product takes bf16 inputs (weights converted when loaded, activations
// rounded to nearest even as they are written to the A tiles) and accumulates in fp32; biases,
// nonlinearities, the reparameterised draws and everything kept between steps stay fp32.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void guide_transition(GuideArgs a) {
    extern __shared__ __align__(16) char lds_raw[];
    const int Zp = a.Zp, Z = a.Z, S = a.S;
    const int Wp = a.Rp > a.Hp ? a.Rp : a.Hp;
    const Lds s = carve<BF16>(lds_raw, Zp, Wp);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int s0 = blockIdx.x * kRows;
    auto put = [](f32x4 *tile, int row, int col, float v) { tile_put<BF16>(tile, kLda, row, col, v); };

    {   // clear the A tiles: pad columns beyond a layer's last 32-block are read by the next layer
        constexpr int PL = BF16 ? 8 : 4;
        const int entries = (2 * (Zp / PL) + Wp / PL) * kLda;
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        for (int i = tid; i < entries; i += kThreads) s.zA[i] = zero;  // zA, hA, mA are contiguous
    }
    __syncthreads();
    for (int idx = tid; idx < kRows * Zp; idx += kThreads) {
        const int row = idx / Zp, c = idx % Zp;
        put(s.zA, row, c, a.z0[c]);
    }
    __syncthreads();

    for (int t = 0; t < a.L; ++t) {
        const float *__restrict__ cf = a.ctx_f + (size_t)t * a.Rp;
        const float *__restrict__ cb = a.ctx_b + (size_t)t * a.Rp;
        wide_layer<BF16>(a.comb, s.zA, wave, lane, [&](int row, int col, float v) {
            put(s.hA, row, col, (tanh_f(v) + cf[col] + cb[col]) * (1.0f / 3.0f));
        });
        __syncthreads();
        narrow_layer<BF16>(a.mu, s.hA, s.red, wave, lane, [&](int row, int col, float v) {
            put(s.mA, row, col, v);
            s.GT[row * Zp + col] = v;  // unrounded mean for the draw
        });
        const float *__restrict__ eq = a.eps_q + (size_t)t * S * Z;
        const bool last = t == a.L - 1;
        wide_layer<BF16>(a.sig, s.mA, wave, lane, [&](int row, int col, float v) {
            const int smp = s0 + row;
            float z = 0.f;
            if (col < Z) {
                const float e = smp < S ? eq[(size_t)smp * Z + col] : 0.f;
                z = s.GT[row * Zp + col] + softplus_f(v) * e;
                if (last && a.z_last && smp < S) a.z_last[(size_t)smp * Z + col] = z;
            }
            put(s.zA, row, col, z);
        });
        __syncthreads();
    }

    // gated transition
    wide_layer<BF16>(a.gate1, s.zA, wave, lane, [&](int row, int col, float v) { put(s.hA, row, col, fmaxf(v, 0.f)); });
    wide_layer<BF16>(a.lin, s.zA, wave, lane, [&](int row, int col, float v) { s.linT[row * Zp + col] = v; });
    __syncthreads();
    narrow_layer<BF16>(a.gate2, s.hA, s.red, wave, lane,
                       [&](int row, int col, float v) { s.gT[row * Zp + col] = sigmoid_f(v); });
    wide_layer<BF16>(a.prop1, s.zA, wave, lane, [&](int row, int col, float v) { put(s.hA, row, col, fmaxf(v, 0.f)); });
    __syncthreads();
    narrow_layer<BF16>(a.prop2, s.hA, s.red, wave, lane, [&](int row, int col, float v) {
        const float g = s.gT[row * Zp + col];
        const float G = col < Z ? (1.f - g) * s.linT[row * Zp + col] + g * v : 0.f;
        s.GT[row * Zp + col] = G;
        put(s.mA, row, col, fmaxf(G, 0.f));
    });
    wide_layer<BF16>(a.tscale, s.mA, wave, lane, [&](int row, int col, float v) {
        const int smp = s0 + row;
        if (smp >= S) return;
        float zn = 0.f;
        if (col < Z) {
            zn = s.GT[row * Zp + col] + softplus_f(v) * a.eps_z[(size_t)smp * Z + col];
            if (a.z_next_dbg) a.z_next_dbg[(size_t)smp * Z + col] = zn;
        }
        a.z_next[(size_t)smp * Zp + col] = zn;
    });
}

}  // namespace

size_t guide_lds_bytes(int Zp, int Rp, int Hp, bool bf16) {
    const int Wp = Rp > Hp ? Rp : Hp;
    const int pl = bf16 ? 8 : 4;
    return (size_t)(2 * (Zp / pl) + Wp / pl) * kLda * 16 + 4 * 1024 * 4 + 3 * (size_t)kRows * Zp * 4;
}

int guide_prepare(int Zp, int Rp, int Hp, bool bf16) {
    const size_t bytes = guide_lds_bytes(Zp, Rp, Hp, bf16);
    if (bytes > 160 * 1024) return DKF_EUNSUPPORTED;
    const void *fn = bf16 ? reinterpret_cast<const void *>(guide_transition<true>)
                          : reinterpret_cast<const void *>(guide_transition<false>);
    DKF_HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    return DKF_OK;
}

int launch_guide(const GuideArgs &a, hipStream_t stream) {
    StageTimer timer(kStageGuide, stream);
    const size_t lds = guide_lds_bytes(a.Zp, a.Rp, a.Hp, a.bf16);
    const dim3 grid((a.S + kRows - 1) / kRows);
    if (a.bf16)
        hipLaunchKernelGGL(guide_transition<true>, grid, dim3(kThreads), lds, stream, a);
    else
        hipLaunchKernelGGL(guide_transition<false>, grid, dim3(kThreads), lds, stream, a);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

}  // namespace dkf
