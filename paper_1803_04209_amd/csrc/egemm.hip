// Emission network in bf16 (Sec. 3.1.3: I = MLP_2(z), J = MLP_2(I(z)), x ~ N(I, J)) as four
// matrix products on operands that are already in matrix-core fragment order.
//
// Every layer is computed transposed, Y^T = W X^T, with v_mfma_f32_32x32x16_bf16: weights are
// the A operand, activations the B operand, so a result tile (lane = sample, 16 features per
// lane) rounded to bf16 is directly two B fragments of the next layer (see gchain.hip for the
// feature order).  A fragment is 1 KiB = 64 lanes x 16 bytes, so producers write and consumers
// read activations with fully coalesced 16-byte accesses and nothing is converted or
// transposed on the way:
//   weights      wfrag[feature block of 32][k-step of 16][lane]
//   activations  xfrag[sample block of 32][k-step of 16][lane]
// A workgroup of four wavefronts (2 x 2) owns 128 or 256 features x 128 samples; fragments of a
// chunk of k-steps are staged once per workgroup in LDS (double buffered) and each wavefront
// multiplies its 2 x 2 or 4 x 2 tiles from there.  The emission mean is kept twice: as bf16
// fragments (input of the scale network) and in fp32 in result-tile order (for the draw).
#include "common.h"
#include "mfma_tile.h"

namespace dkf {
namespace {

constexpr int kThreads = 256;
constexpr int kMeanStride = 36;               // floats per row of the epilogue's transposition tile (16-byte aligned rows)

template <int G>
__device__ __forceinline__ f32x4 pack_half(const f32x16 &v) {  // half G of a result tile as a B fragment
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = (__bf16)v[8 * G + j];
    return __builtin_bit_cast(f32x4, r);
}

// TM x 2 tiles of 32 x 32 per wavefront (features x samples), 2 x 2 wavefronts: a workgroup owns
// 64 TM features x 128 samples.  What bounds the main loop is LDS read bandwidth (measured: with the
// global loads and LDS writes taken out the 2 x 2 variant still runs at 38 % of the matrix rate):
// every 32 x 32 x 16 instruction consumes two 1 KiB fragments, and a wavefront with TM x TN tiles
// reads TM + TN fragments per TM * TN instructions -- 32 bytes per clock at 2 x 2, which for four
// SIMDs is all the LDS has; 4 x 2 needs 24 (and a quarter less from L2).
//   TM = 2: the H-wide layers (a 4 x 2 tiling would leave half the compute units without work there)
//   TM = 4: the N-wide layers
// A chunk is KC k-steps = 32 (TM = 2) or 24 (TM = 4) fragments; kDepth chunks are in flight in
// registers.  (4 x 4 tiles would halve the LDS reads again, but their 256 accumulator registers per
// lane leave hipcc spilling inside the main loop: measured 6x slower.)
template <int EPI, int TM>
__global__ __launch_bounds__(kThreads, 2) void frag_gemm(FragGemmArgs a) {
    constexpr int TN = 2, kFeatBlocks = 2 * TM, kSampBlocks = 2 * TN, KC = TM == 2 ? 4 : 2;
    constexpr int kChunkFrags = (kFeatBlocks + kSampBlocks) * KC, kFragsPerWave = kChunkFrags / 4;
    constexpr int kDepth = TM == 2 ? 4 : 2;
    static_assert(kChunkFrags % 4 == 0 && 4 * 32 * kMeanStride * 4 <= kChunkFrags * 1024, "chunk size");
    __shared__ f32x4 lds[2][kChunkFrags * 64];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wf = wave >> 1, ws = wave & 1;
    // workgroups that share a sample tile run on the same XCD (consecutive ids are dealt
    // round-robin to the 8 XCDs), so its activation fragments are fetched into one L2 only
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int samp_tile = xcd + 8 * (seq / a.feat_tiles);
    const int feat_tile = seq % a.feat_tiles;
    if (samp_tile >= a.samp_tiles) return;
    const int KS = a.k_steps, n_chunks = KS / KC;
    const f32x4 *__restrict__ W = reinterpret_cast<const f32x4 *>(a.wfrag);
    const f32x4 *__restrict__ X = reinterpret_cast<const f32x4 *>(a.xfrag);

    // fragment j of a chunk: j < kFeatBlocks * KC -> weights (block j / KC, k-step j % KC), else activations
    const f32x4 *src[kFragsPerWave];
#pragma unroll
    for (int i = 0; i < kFragsPerWave; ++i) {
        const int j = wave * kFragsPerWave + i;
        if (j < kFeatBlocks * KC) {
            src[i] = W + ((size_t)(feat_tile * kFeatBlocks + j / KC) * KS + j % KC) * 64 + lane;
        } else {
            const int jj = j - kFeatBlocks * KC;
            src[i] = X + ((size_t)(samp_tile * kSampBlocks + jj / KC) * KS + jj % KC) * 64 + lane;
        }
    }

    // The last layer's result is not an operand of anything, so it is computed the other way round
    // (activations as the A operand): a lane then owns one feature and 16 samples, and the noise
    // reads and sample writes of its epilogue are 128 contiguous bytes per row.
    constexpr bool kRowsAreSamples = EPI == kFragDraw;
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int mb = feat_tile * kFeatBlocks + wf * TM + i;
        f32x16 v;
        if constexpr (kRowsAreSamples) {
            const float b = a.bias[32 * mb + (lane & 31)];
#pragma unroll
            for (int e = 0; e < 16; ++e) v[e] = b;
        } else {
            const float *b = a.bias + 32 * mb + 4 * (lane >> 5);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 bq = *reinterpret_cast<const f32x4 *>(b + 8 * q);
                v[4 * q] = bq[0]; v[4 * q + 1] = bq[1]; v[4 * q + 2] = bq[2]; v[4 * q + 3] = bq[3];
            }
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = v;
    }

    // Fragments travel global -> registers -> LDS.  kDepth chunks are in flight in registers, so
    // that a chunk's load latency is covered by the matrix work of the chunks before it (one
    // workgroup per compute unit has nothing else to hide it behind); LDS is double buffered.
    f32x4 stage[kDepth][kFragsPerWave];
    // (Past the end the last chunk is fetched again and staged into the idle buffer: keeping the
    // loop free of data-dependent branches lets every wait name exactly the loads it needs.)
    auto issue = [&](int d, int chunk) {
        const int ch = chunk < n_chunks ? chunk : n_chunks - 1;
        // scheduling fences: loads return in issue order, so a chunk's loads must stay together and
        // behind those of the chunks before it, or the wait for them also waits for younger ones
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kFragsPerWave; ++i) stage[d][i] = src[i][(size_t)ch * KC * 64];
        __builtin_amdgcn_sched_barrier(0);
    };
    auto to_lds = [&](int d, int buf) {
#pragma unroll
        for (int i = 0; i < kFragsPerWave; ++i) lds[buf][(wave * kFragsPerWave + i) * 64 + lane] = stage[d][i];
    };
#pragma unroll
    for (int d = 0; d < kDepth; ++d) issue(d, d);
    to_lds(0, 0);
    issue(0, kDepth);
    __syncthreads();

    const f32x4 *A0 = &lds[0][(wf * TM * KC) * 64 + lane];
    const f32x4 *B0 = &lds[0][((kFeatBlocks + ws * TN) * KC) * 64 + lane];
    // (unrolled twice over the register ring: the compiler's wait at the loop head is for all loads)
    for (int c0 = 0; c0 < n_chunks; c0 += 2 * kDepth) {
#pragma unroll
        for (int d = 0; d < 2 * kDepth; ++d) {
            const int c = c0 + d;
            if (c >= n_chunks) break;
            const f32x4 *A = A0 + (d & 1) * kChunkFrags * 64, *B = B0 + (d & 1) * kChunkFrags * 64;  // kDepth is even
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                bf16x8 wa[TM], xb[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) wa[i] = __builtin_bit_cast(bf16x8, A[(i * KC + k) * 64]);
#pragma unroll
                for (int j = 0; j < TN; ++j) xb[j] = __builtin_bit_cast(bf16x8, B[(j * KC + k) * 64]);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = kRowsAreSamples
                                        ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(xb[j], wa[i], acc[i][j], 0, 0, 0)
                                        : __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[i], xb[j], acc[i][j], 0, 0, 0);
            }
            // the next chunk has been in registers for kDepth - 1 chunks of work
            to_lds((d + 1) % kDepth, (d + 1) & 1);
            issue((d + 1) % kDepth, c + 1 + kDepth);
            __syncthreads();
        }
    }

    // ---- epilogue ----------------------------------------------------------------------
    const int h = lane >> 5;
    float scale = 1.f;
    if constexpr (EPI == kFragDraw) scale = a.ctl->scale;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int mb = feat_tile * kFeatBlocks + wf * TM + i;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int sb = samp_tile * kSampBlocks + ws * TN + j;
            f32x16 &v = acc[i][j];
            if constexpr (EPI == kFragRelu) {
#pragma unroll
                for (int e = 0; e < 16; ++e) v[e] = fmaxf(v[e], 0.f);
            }
            if constexpr (EPI != kFragDraw) {
                f32x4 *out = reinterpret_cast<f32x4 *>(a.out_frag) + ((size_t)sb * a.out_k_steps + 2 * mb) * 64 + lane;
                out[0] = pack_half<0>(v);
                out[64] = pack_half<1>(v);
            }
            if constexpr (EPI == kFragMean) {
                f32x4 *out = reinterpret_cast<f32x4 *>(a.mean_tiles) + ((size_t)sb * a.out_k_steps / 2 + mb) * 4 * 64 + lane;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 m = {v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]};
                    out[q * 64] = m;
                }
            }
            if constexpr (EPI == kFragDraw) {
                // the mean's tile is stored with lanes along samples: turn it through a wavefront-private
                // LDS tile (the staging buffers are free by now) so that m[e] belongs to acc element e
                float *tile = reinterpret_cast<float *>(&lds[0][0]) + wave * (32 * kMeanStride);
                const f32x4 *mt = reinterpret_cast<const f32x4 *>(a.mean_tiles) + ((size_t)sb * a.mean_blocks + mb) * 4 * 64 + lane;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<f32x4 *>(tile + (lane & 31) * kMeanStride + 8 * q + 4 * h) = mt[q * 64];
                float m[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) m[e] = tile[(8 * (e >> 2) + 4 * h + (e & 3)) * kMeanStride + (lane & 31)];
                const int N = a.N, f = 32 * mb + (lane & 31);
                const float *__restrict__ eps_x = a.eps_x;
                float eps[16];  // all of the tile's noise requested before the first store
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int smp = sb * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
                    eps[e] = (smp < a.S && f < N) ? eps_x[(size_t)smp * N + f] : 0.f;
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int smp = sb * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
                    if (smp >= a.S || f >= N) continue;
                    const size_t at = (size_t)smp * N + f;
                    const float sd = softplus_f(v[e]);
                    a.out_samples[at] = scale * (m[e] + sd * eps[e]);
                    if (a.out_mean_dbg) a.out_mean_dbg[at] = m[e];
                    if (a.out_sd_dbg) a.out_sd_dbg[at] = sd;
                }
            }
        }
    }
}

template <int TM>
void launch_t(const FragGemmArgs &a, dim3 grid, hipStream_t stream) {
    switch (a.epilogue) {
        case kFragIdentity: hipLaunchKernelGGL((frag_gemm<kFragIdentity, TM>), grid, dim3(kThreads), 0, stream, a); break;
        case kFragRelu: hipLaunchKernelGGL((frag_gemm<kFragRelu, TM>), grid, dim3(kThreads), 0, stream, a); break;
        case kFragMean: hipLaunchKernelGGL((frag_gemm<kFragMean, TM>), grid, dim3(kThreads), 0, stream, a); break;
        default: hipLaunchKernelGGL((frag_gemm<kFragDraw, TM>), grid, dim3(kThreads), 0, stream, a); break;
    }
}

}  // namespace

// feat_tiles counts tiles of 64 * a.tile features, samp_tiles tiles of 128 samples
int launch_frag_gemm(const FragGemmArgs &a, int stage, hipStream_t stream) {
    if (a.tile != 2 && a.tile != 4) return DKF_EUNSUPPORTED;
    if (a.epilogue < kFragIdentity || a.epilogue > kFragDraw) return DKF_EINVAL;
    if (a.k_steps < 4 || a.k_steps % 4 != 0 || a.feat_tiles < 1 || a.samp_tiles < 1) return DKF_EINVAL;
    if (a.epilogue == kFragDraw &&
        ((reinterpret_cast<uintptr_t>(a.eps_x) | reinterpret_cast<uintptr_t>(a.out_samples) |
          reinterpret_cast<uintptr_t>(a.out_mean_dbg) | reinterpret_cast<uintptr_t>(a.out_sd_dbg)) & 15))
        return DKF_EINVAL;
    StageTimer timer(stage, stream);
    const int samp_tiles8 = (a.samp_tiles + 7) / 8 * 8;
    const dim3 grid(samp_tiles8 * a.feat_tiles);
    if (a.tile == 2) launch_t<2>(a, grid, stream);
    else launch_t<4>(a, grid, stream);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

}  // namespace dkf
