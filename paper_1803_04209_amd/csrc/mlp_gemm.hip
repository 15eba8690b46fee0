// Dense layers of the emission network over all S samples (Sec. 3.1.3):
//   I(z) = W_I2 act(W_I1 z + b) + b          (mean, N wide)
//   J(z) = softplus(W_J2 relu(W_J1 I(z) + b) + b)   (scale, fed by the mean)
//   x    = s * (I + J * eps_x)                 (draw, back in seconds)
// One kernel template computes  out[S][n] = epilogue(A[S][K] W^T + b)  on the
// fp32 matrix cores: a workgroup owns a 128 x 128 output tile, each of its four
// wavefronts a 64 x 64 quarter (2 x 2 MFMA blocks).  The activation tile is
// staged through LDS in K chunks of 32 (double buffered); the weights are read
// straight from L2 in the pre-tiled PackedLayer order and prefetched one chunk
// ahead in registers.  The scale layer's epilogue applies softplus, mixes in
// the noise and writes the sample, so J is never materialised.
#include "common.h"
#include "mfma_tile.h"

namespace dkf {
namespace {

constexpr int kThreads = 256;
constexpr int kTileM = 128;
constexpr int kTileNB = 4;            // 32-column blocks per workgroup
constexpr int kChunkKG = 4;           // k-groups per LDS chunk: K chunk = 32 columns in fp32, 64 in bf16
constexpr int kLda = kTileM + 1;      // plane stride in 16-byte entries
constexpr int kPlanes = kChunkKG * 2; // planes per chunk (4 fp32 or 8 bf16 columns each)

// BF16: the activation rows are read as fp32 and rounded to bf16 (nearest even) while they are
// staged into LDS; the layer's tiles are bf16; accumulation and the epilogue stay fp32.
template <int EPI, bool BF16>
__global__ __launch_bounds__(kThreads, 2) void mlp_gemm(GemmArgs a) {
    __shared__ f32x4 As[2][kPlanes * kLda];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n_col_tiles = (a.layer.n_blocks + kTileNB - 1) / kTileNB;
    // Workgroups that share a row tile run on the same XCD (consecutive ids are
    // dealt round-robin to the 8 XCDs), so the activation rows are fetched into
    // one L2 only.
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int row_tile = xcd + 8 * (seq / n_col_tiles);
    const int col_tile = seq % n_col_tiles;
    const int m0 = row_tile * kTileM;
    if (m0 >= a.S) return;

    const int wr = wave >> 1, wc = wave & 1;
    const int KG = a.layer.k_groups;
    const int n_chunks = KG / kChunkKG;
    int nb[2];
    const f32x4 *bt[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        nb[j] = col_tile * kTileNB + wc * 2 + j;
        const int nbc = nb[j] < a.layer.n_blocks ? nb[j] : a.layer.n_blocks - 1;
        bt[j] = reinterpret_cast<const f32x4 *>(a.layer.tiles) + (size_t)nbc * KG * 64 + lane;
    }

    // global -> LDS mapping of the activation chunk: plane q = tid % 8, rows tid/8 + 32 i
    constexpr int kPlaneCols = BF16 ? 8 : 4;  // columns per plane
    constexpr int kLoads = BF16 ? 2 : 1;      // float4 loads per plane entry
    const int lq = tid & 7, lrow = tid >> 3;
    const float *arow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = m0 + lrow + 32 * i;
        if (r >= a.S) r = a.S - 1;
        arow[i] = a.A + (size_t)r * a.lda + lq * kPlaneCols;
    }
    auto stage = [](const f32x4 (&v)[kLoads]) {  // one 16-byte plane entry from kLoads float4
        if constexpr (BF16) {
            bf16x8 h;
#pragma unroll
            for (int e = 0; e < 4; ++e) { h[e] = (__bf16)v[0][e]; h[4 + e] = (__bf16)v[1][e]; }
            return __builtin_bit_cast(f32x4, h);
        } else {
            return v[0];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = zero16();

    f32x4 areg[4][kLoads];
    f32x4 breg[2][kChunkKG];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int l = 0; l < kLoads; ++l) areg[i][l] = *reinterpret_cast<const f32x4 *>(arow[i] + 4 * l);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int g = 0; g < kChunkKG; ++g) breg[j][g] = bt[j][(size_t)g * 64];
#pragma unroll
    for (int i = 0; i < 4; ++i) As[0][lq * kLda + lrow + 32 * i] = stage(areg[i]);
    __syncthreads();

    const int r = lane & 31, half = lane >> 5;
    for (int ch = 0; ch < n_chunks; ++ch) {
        const int cur = ch & 1;
        f32x4 bcur[2][kChunkKG];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int g = 0; g < kChunkKG; ++g) bcur[j][g] = breg[j][g];
        const bool more = ch + 1 < n_chunks;
        if (more) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int l = 0; l < kLoads; ++l)
                    areg[i][l] = *reinterpret_cast<const f32x4 *>(arow[i] + (size_t)(ch + 1) * kPlanes * kPlaneCols + 4 * l);
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int g = 0; g < kChunkKG; ++g)
                    breg[j][g] = bt[j][(size_t)((ch + 1) * kChunkKG + g) * 64];
        }
#pragma unroll
        for (int g = 0; g < kChunkKG; ++g) {
            const f32x4 a0 = As[cur][(g * 2 + half) * kLda + wr * 64 + r];
            const f32x4 a1 = As[cur][(g * 2 + half) * kLda + wr * 64 + 32 + r];
            if constexpr (BF16) {
                acc[0][0] = mfma32_bf16(a0, bcur[0][g], acc[0][0]);
                acc[0][1] = mfma32_bf16(a0, bcur[1][g], acc[0][1]);
                acc[1][0] = mfma32_bf16(a1, bcur[0][g], acc[1][0]);
                acc[1][1] = mfma32_bf16(a1, bcur[1][g], acc[1][1]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[0][0] = mfma32(a0[e], bcur[0][g][e], acc[0][0]);
                    acc[0][1] = mfma32(a0[e], bcur[1][g][e], acc[0][1]);
                    acc[1][0] = mfma32(a1[e], bcur[0][g][e], acc[1][0]);
                    acc[1][1] = mfma32(a1[e], bcur[1][g][e], acc[1][1]);
                }
            }
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < 4; ++i) As[cur ^ 1][lq * kLda + lrow + 32 * i] = stage(areg[i]);
        }
        __syncthreads();
    }

    // epilogue.  The draw reads two values per result: all of a tile's reads are requested, from
    // clamped addresses, before the first value is used (a read behind a branch is waited for
    // where the branch joins, one memory round trip per element).
    float scale = 1.f;
    if constexpr (EPI == kEpiScaleDraw) scale = a.ctl->scale;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if (nb[j] >= a.layer.n_blocks) continue;
        const int col = nb[j] * 32 + r;
        const float b = a.layer.bias[col];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if constexpr (EPI == kEpiScaleDraw) {
                const float *__restrict__ mean_in = a.mean;
                const float *__restrict__ eps_in = a.eps_x;
                const int cc = col < a.N ? col : a.N - 1;
                float mean[16], eps[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wr * 64 + i * 32 + acc_row(e, lane);
                    const int rc = row < a.S ? row : a.S - 1;
                    mean[e] = mean_in[(size_t)rc * a.ld_mean + cc];
                    eps[e] = eps_in[(size_t)rc * a.N + cc];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wr * 64 + i * 32 + acc_row(e, lane);
                    if (row >= a.S || col >= a.N) continue;
                    const float sd = softplus_f(acc[i][j][e] + b);
                    a.out_samples[(size_t)row * a.N + col] = scale * (mean[e] + sd * eps[e]);
                    if (a.out_mean_dbg) a.out_mean_dbg[(size_t)row * a.N + col] = mean[e];
                    if (a.out_sd_dbg) a.out_sd_dbg[(size_t)row * a.N + col] = sd;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wr * 64 + i * 32 + acc_row(e, lane);
                    if (row >= a.S) continue;
                    const float v = acc[i][j][e] + b;
                    a.out[(size_t)row * a.ldo + col] = EPI == kEpiBiasRelu ? fmaxf(v, 0.f) : v;
                }
            }
        }
    }
}

}  // namespace

int launch_gemm(const GemmArgs &a, int stage, hipStream_t stream) {
    if (a.layer.k_groups % kChunkKG != 0 || a.layer.k_groups * (a.bf16 ? 16 : 8) > a.lda) return DKF_EINVAL;
    StageTimer timer(stage, stream);
    const int row_tiles = (a.S + kTileM - 1) / kTileM;
    const int col_tiles = (a.layer.n_blocks + kTileNB - 1) / kTileNB;
    const int row_tiles8 = (row_tiles + 7) / 8 * 8;
    const dim3 grid(row_tiles8 * col_tiles);
#define DKF_GEMM_LAUNCH(E_)                                                                       \
    if (a.bf16) hipLaunchKernelGGL((mlp_gemm<E_, true>), grid, dim3(kThreads), 0, stream, a);    \
    else hipLaunchKernelGGL((mlp_gemm<E_, false>), grid, dim3(kThreads), 0, stream, a);          \
    break
    switch (a.epilogue) {
        case kEpiBias: DKF_GEMM_LAUNCH(kEpiBias);
        case kEpiBiasRelu: DKF_GEMM_LAUNCH(kEpiBiasRelu);
        case kEpiScaleDraw: DKF_GEMM_LAUNCH(kEpiScaleDraw);
        default: return DKF_EINVAL;
    }
#undef DKF_GEMM_LAUNCH
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

}  // namespace dkf
