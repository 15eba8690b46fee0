// Emission network in bf16 (Sec. 3.1.3: I = MLP_2(z), J = MLP_2(I(z)), x ~ N(I, J)) as matrix
// products on operands that are already in matrix-core fragment order.
//
// Every layer is computed transposed, Y^T = W X^T, with v_mfma_f32_32x32x16_bf16: weights are
// the A operand, activations the B operand, so a result tile (lane = sample, 16 features per
// lane) rounded to bf16 is directly two B fragments of the next layer (see gchain.hip for the
// feature order).  A fragment is 1 KiB = 64 lanes x 16 bytes, so producers write and consumers
// read activations with fully coalesced 16-byte accesses and nothing is converted or
// transposed on the way:
//   weights      wfrag[feature block of 32][k-step of 16][lane]
//   activations  xfrag[sample block of 32][k-step of 16][lane]
// A workgroup of four wavefronts owns 64 or 128 features x 256 samples, each wavefront 64 of the
// samples; weight fragments are staged once per workgroup in LDS, activation fragments go straight
// into the registers of the wavefront that multiplies them.
//
// The mean I(z) ends in a linear layer and J's first layer is linear in I, so the N-wide vector
// between them never has to exist: with M = W_J1 W_I2 (H x H) and c = W_J1 b_I2 + b_J1, formed once
// when the weights are loaded, J's hidden layer is relu(M h + c) on the mean's hidden layer h.
// Three launches: h, J's hidden layer, and one kernel that multiplies both N-wide output layers
// for the same tile of (sample, worker) pairs and draws x from them -- neither the mean nor the
// scale is ever written to memory.
#include "common.h"
#include "mfma_tile.h"

namespace dkf {
namespace {

constexpr int kThreads = 256;
constexpr int kTN = 2;   // sample blocks per wavefront
constexpr int kKC = 4;   // k-steps per chunk of weights staged in LDS

template <int G>
__device__ __forceinline__ f32x4 pack_half(const f32x16 &v) {  // half G of a result tile as a B fragment
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = (__bf16)v[8 * G + j];
    return __builtin_bit_cast(f32x4, r);
}

// acc[i][j] = bias + W X^T for TM feature blocks x kTN sample blocks of 32 (or its transpose, lanes
// along the features, when ROWS_ARE_SAMPLES: the two operands swap roles, the same bytes serve);
// with ADD the product is added to what acc holds and bias is not read.
// What bounds a product of fragments is operand delivery, not the matrix cores: a 32 x 32 x 16
// instruction consumes two 1 KiB fragments in 32 clocks, LDS delivers at most 128 bytes per clock
// to the four SIMDs together and the vector memory path 64.  So the two operands take different
// roads.  Weights are shared by all four wavefronts: staged once per workgroup in LDS (double
// buffered, a chunk of kKC k-steps at a time) and read by each wavefront, TM fragments per
// TM * kTN instructions.  Activations belong to one wavefront only: they go from memory straight
// into its registers, DEPTH chunks ahead, and never touch LDS.  Per instruction that is 5/8 KiB of
// LDS traffic and 1/4 KiB (TM = 4) or 1/2 KiB (TM = 2) of loads, against 9/8 KiB of LDS traffic
// when both operands are staged for 2 x 2 wavefronts.  (4 x 4 tiles would halve the LDS reads
// again, but their 256 accumulator registers per lane leave hipcc spilling inside the main loop:
// measured 6x slower.)
// All four wavefronts of the workgroup must call this together (it holds barriers); lds is two
// buffers of BUF fragments, BUF >= TM * kKC.
template <int TM, int DEPTH, bool ROWS_ARE_SAMPLES, int BUF, bool ADD = false>
__device__ __forceinline__ void product(const float *wfrag, const float *xfrag, const float *bias, int KS,
                                        int feat_block0, int samp_block0, f32x4 *lds, f32x16 (&acc)[TM][kTN]) {
    constexpr int kChunkFrags = TM * kKC, kFragsPerWave = kChunkFrags / 4;
    constexpr int kUnroll = 8;  // chunks per trip of the main loop (even, a multiple of DEPTH)
    static_assert(BUF >= kChunkFrags && kUnroll % 2 == 0 && kUnroll % DEPTH == 0, "buffers");
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n_chunks = KS / kKC;
    const f32x4 *__restrict__ W = reinterpret_cast<const f32x4 *>(wfrag);
    const f32x4 *__restrict__ X = reinterpret_cast<const f32x4 *>(xfrag);

    // weight fragment j of a chunk is (feature block j / kKC, k-step j % kKC); this wavefront stages
    // fragments wave * kFragsPerWave ...
    const f32x4 *wsrc[kFragsPerWave];
#pragma unroll
    for (int i = 0; i < kFragsPerWave; ++i) {
        const int j = wave * kFragsPerWave + i;
        wsrc[i] = W + ((size_t)(feat_block0 + j / kKC) * KS + j % kKC) * 64 + lane;
    }
    // ... and multiplies its own kTN sample blocks
    const f32x4 *xsrc[kTN];
#pragma unroll
    for (int j = 0; j < kTN; ++j) xsrc[j] = X + (size_t)(samp_block0 + j) * KS * 64 + lane;

#pragma unroll
    for (int i = 0; i < (ADD ? 0 : TM); ++i) {
        const int mb = feat_block0 + i;
        f32x16 v;
        if constexpr (ROWS_ARE_SAMPLES) {
            const float b = bias[32 * mb + (lane & 31)];
#pragma unroll
            for (int e = 0; e < 16; ++e) v[e] = b;
        } else {
            const float *b = bias + 32 * mb + 4 * (lane >> 5);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 bq = *reinterpret_cast<const f32x4 *>(b + 8 * q);
                v[4 * q] = bq[0]; v[4 * q + 1] = bq[1]; v[4 * q + 2] = bq[2]; v[4 * q + 3] = bq[3];
            }
        }
#pragma unroll
        for (int j = 0; j < kTN; ++j) acc[i][j] = v;
    }

    // Loads return in issue order and every wait names how many younger loads may stay in flight,
    // so the order of issue is fixed by scheduling fences: in trip c the activations of chunk
    // c + DEPTH follow the instructions that consumed their registers, k-step by k-step, and the
    // weights of chunk c + 2 follow the copy of chunk c + 1 into LDS.  (Past the end the last chunk
    // is fetched again: a loop free of data-dependent branches keeps those counts exact.)
    f32x4 wstage[kFragsPerWave];
    f32x4 xring[DEPTH][kKC][kTN];
    auto issue_w = [&](int chunk) {
        const int ch = chunk < n_chunks ? chunk : n_chunks - 1;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kFragsPerWave; ++i) wstage[i] = wsrc[i][(size_t)ch * kKC * 64];
        __builtin_amdgcn_sched_barrier(0);
    };
    auto issue_x = [&](int d, int k, int chunk) {
        const int ch = chunk < n_chunks ? chunk : n_chunks - 1;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < kTN; ++j) xring[d][k][j] = xsrc[j][(size_t)(ch * kKC + k) * 64];
        __builtin_amdgcn_sched_barrier(0);
    };
    auto to_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kFragsPerWave; ++i) lds[(buf * BUF + wave * kFragsPerWave + i) * 64 + lane] = wstage[i];
    };
    issue_w(0);
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
#pragma unroll
        for (int k = 0; k < kKC; ++k) issue_x(d, k, d);
    to_lds(0);
    issue_w(1);
    __syncthreads();

    for (int c0 = 0; c0 < n_chunks; c0 += kUnroll) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int c = c0 + u;
            if (c >= n_chunks) break;
            const f32x4 *A = lds + (u & 1) * BUF * 64 + lane;
#pragma unroll
            for (int k = 0; k < kKC; ++k) {
                bf16x8 wa[TM], xb[kTN];
#pragma unroll
                for (int i = 0; i < TM; ++i) wa[i] = __builtin_bit_cast(bf16x8, A[(i * kKC + k) * 64]);
#pragma unroll
                for (int j = 0; j < kTN; ++j) xb[j] = __builtin_bit_cast(bf16x8, xring[u % DEPTH][k][j]);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < kTN; ++j)
                        acc[i][j] = ROWS_ARE_SAMPLES
                                        ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(xb[j], wa[i], acc[i][j], 0, 0, 0)
                                        : __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[i], xb[j], acc[i][j], 0, 0, 0);
                issue_x(u % DEPTH, k, c + DEPTH);
            }
            // (the barrier at the end of the trip before this one freed the other buffer)
            to_lds((u + 1) & 1);
            issue_w(c + 2);
            __syncthreads();
        }
    }
}

// blockIdx -> (feature tile, sample tile): workgroups that share a sample tile run on the same XCD
// (consecutive ids are dealt round-robin to the 8 XCDs), so its activation fragments are fetched
// into one L2 only.  False if this workgroup has no tile.
__device__ __forceinline__ bool tile_of_block(const FragGemmArgs &a, int &feat_tile, int &samp_tile) {
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    samp_tile = xcd + 8 * (seq / a.feat_tiles);
    feat_tile = seq % a.feat_tiles;
    return samp_tile < a.samp_tiles;
}

// One hidden layer: act(W x + b) -> bf16 fragments of the next layer.  32 TM features x 256 samples
// per workgroup.
template <int EPI, int TM>
__global__ __launch_bounds__(kThreads, 2) void frag_gemm(FragGemmArgs a) {
    constexpr int kBuf = TM * kKC;
    __shared__ f32x4 lds[2 * kBuf * 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int feat_tile, samp_tile;
    if (!tile_of_block(a, feat_tile, samp_tile)) return;
    f32x16 acc[TM][kTN];
    product<TM, TM == 2 ? 2 : 1, false, kBuf>(a.wfrag, a.xfrag, a.bias, a.k_steps, feat_tile * TM,
                                             samp_tile * 4 * kTN + wave * kTN, lds, acc);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int mb = feat_tile * TM + i;
#pragma unroll
        for (int j = 0; j < kTN; ++j) {
            const int sb = samp_tile * 4 * kTN + wave * kTN + j;
            f32x16 &v = acc[i][j];
            if constexpr (EPI == kFragRelu) {
#pragma unroll
                for (int e = 0; e < 16; ++e) v[e] = fmaxf(v[e], 0.f);
            }
            f32x4 *out = reinterpret_cast<f32x4 *>(a.out_frag) + ((size_t)sb * a.out_k_steps + 2 * mb) * 64 + lane;
            out[0] = pack_half<0>(v);
            out[64] = pack_half<1>(v);
        }
    }
}

// Both output layers of the emission for one tile and the draw (Sec. 3.1.3):
//   mean = W_I2 h + b_I2,  sd = softplus(W_J2 h' + b_J2),  x = s (mean + sd eps).
// The results are nobody's operand, so they are computed the other way round (activation fragments
// as the A operand): a lane then owns one worker and 16 samples, and the noise reads and sample
// writes are 128 contiguous bytes per row.  64 workers x 256 samples per workgroup.
template <bool DBG>  // DBG: the mean and the scale are written out too
__global__ __launch_bounds__(kThreads, 2) void frag_draw(FragGemmArgs a) {
    constexpr int TM = 2, kBuf = TM * kKC;
    __shared__ f32x4 lds[2 * kBuf * 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int feat_tile, samp_tile;
    if (!tile_of_block(a, feat_tile, samp_tile)) return;
    const int sb0 = samp_tile * 4 * kTN + wave * kTN;
    f32x16 mean[TM][kTN], acc[TM][kTN];
    product<TM, 1, true, kBuf>(a.wfrag2, a.xfrag2, a.bias2, a.k_steps, feat_tile * TM, sb0, lds, mean);
    product<TM, 1, true, kBuf>(a.wfrag, a.xfrag, a.bias, a.k_steps, feat_tile * TM, sb0, lds, acc);

    // The draw moves 8 bytes per result and computes little: what it needs is many loads in flight.
    // All of the wavefront's noise (four tiles, 64 loads of two 128-byte rows each) is requested
    // before the first value is used; the registers of the products' operands are free by now.
    // Stores count in the same in-order counter as loads, and a wait placed where control flow
    // joins is a wait for everything: so the common case (whole tiles, no stage outputs) is
    // straight-line code, selected per wavefront.
    const int h = lane >> 5, N = a.N;
    const float scale = a.ctl->scale;
    const float *__restrict__ eps_x = a.eps_x;
    float *__restrict__ out_samples = a.out_samples;
    const int f0 = 32 * feat_tile * TM + (lane & 31), s00 = sb0 * 32 + 4 * h;
    const bool whole = 32 * (feat_tile + 1) * TM <= N && (sb0 + kTN) * 32 <= a.S;
    if (!DBG && whole) {
        const float *src = eps_x + (size_t)s00 * N + f0;
        float *dst = out_samples + (size_t)s00 * N + f0;
        float eps[TM][kTN][16];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < kTN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) eps[i][j][e] = src[(size_t)(32 * j + 8 * (e >> 2) + (e & 3)) * N + 32 * i];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < kTN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    dst[(size_t)(32 * j + 8 * (e >> 2) + (e & 3)) * N + 32 * i] =
                        scale * (mean[i][j][e] + softplus_f(acc[i][j][e]) * eps[i][j][e]);
        return;
    }
    // ragged tiles and stage outputs: the same with the noise read from clamped addresses (no branch
    // between a load and its use) and guarded stores
    const int f_last = N - 1, s_last = a.S - 1;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int f = f0 + 32 * i;
#pragma unroll
        for (int j = 0; j < kTN; ++j) {
            float eps[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int smp = s00 + 32 * j + 8 * (e >> 2) + (e & 3);
                eps[e] = eps_x[(size_t)(smp < s_last ? smp : s_last) * N + (f < f_last ? f : f_last)];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int smp = s00 + 32 * j + 8 * (e >> 2) + (e & 3);
                if (smp >= a.S || f >= N) continue;
                const size_t at = (size_t)smp * N + f;
                const float sd = softplus_f(acc[i][j][e]);
                out_samples[at] = scale * (mean[i][j][e] + sd * eps[e]);
                if (DBG && a.out_mean_dbg) a.out_mean_dbg[at] = mean[i][j][e];
                if (DBG && a.out_sd_dbg) a.out_sd_dbg[at] = sd;
            }
        }
    }
}

// The same for launches made of whole tiles that ask for no stage outputs, 128 workers x 256
// samples per workgroup.  Only one set of accumulators is alive at a time: the scale's product comes
// first, each of its results is replaced in place by b_I2 + softplus(.) eps, and the mean's product is
// added on top of that, so what is left to do after the second product is one multiplication and
// the store.  That halves the registers, which pays for result tiles twice as large (half the LDS
// reads per instruction), and puts the noise loads between two stretches of matrix work.
__global__ __launch_bounds__(kThreads, 2) void frag_draw_whole(FragGemmArgs a) {
    constexpr int TM = 4, kBuf = TM * kKC;
    __shared__ f32x4 lds[2 * kBuf * 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int feat_tile, samp_tile;
    if (!tile_of_block(a, feat_tile, samp_tile)) return;
    const int sb0 = samp_tile * 4 * kTN + wave * kTN;
    f32x16 acc[TM][kTN];
    product<TM, 1, true, kBuf>(a.wfrag, a.xfrag, a.bias, a.k_steps, feat_tile * TM, sb0, lds, acc);

    const int N = a.N;
    const size_t at0 = (size_t)(sb0 * 32 + 4 * (lane >> 5)) * N + 32 * feat_tile * TM + (lane & 31);
    const float *__restrict__ src = a.eps_x + at0;
    const float *__restrict__ b_mean = a.bias2 + 32 * feat_tile * TM + (lane & 31);
    // (half of the tiles at a time: 64 loads in flight per wavefront)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        float eps[2][kTN][16];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < kTN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    eps[i][j][e] = src[(size_t)(32 * j + 8 * (e >> 2) + (e & 3)) * N + 32 * (2 * half + i)];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const float b = b_mean[32 * (2 * half + i)];
#pragma unroll
            for (int j = 0; j < kTN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    acc[2 * half + i][j][e] = b + softplus_f(acc[2 * half + i][j][e]) * eps[i][j][e];
        }
    }
    product<TM, 1, true, kBuf, true>(a.wfrag2, a.xfrag2, nullptr, a.k_steps, feat_tile * TM, sb0, lds, acc);

    const float scale = a.ctl->scale;
    float *__restrict__ dst = a.out_samples + at0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < kTN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                dst[(size_t)(32 * j + 8 * (e >> 2) + (e & 3)) * N + 32 * i] = scale * acc[i][j][e];
}

template <int TM>
void launch_t(const FragGemmArgs &a, dim3 grid, hipStream_t stream) {
    if (a.epilogue == kFragRelu) hipLaunchKernelGGL((frag_gemm<kFragRelu, TM>), grid, dim3(kThreads), 0, stream, a);
    else hipLaunchKernelGGL((frag_gemm<kFragIdentity, TM>), grid, dim3(kThreads), 0, stream, a);
}

}  // namespace

// feat_tiles counts tiles of 32 * a.tile features, samp_tiles tiles of 256 samples.  For the draw the
// tiling is chosen here (tile and feat_tiles are not read): whole-tile launches without stage
// outputs take the kernel with 128-worker tiles, everything else the one with 64-worker tiles.
int launch_frag_gemm(const FragGemmArgs &a, int stage, hipStream_t stream) {
    const bool draw = a.epilogue == kFragDraw;
    if (!draw && a.tile != 2 && a.tile != 4) return DKF_EUNSUPPORTED;
    if (a.epilogue < kFragIdentity || a.epilogue > kFragDraw) return DKF_EINVAL;
    if (a.k_steps < 4 || a.k_steps % 4 != 0 || a.samp_tiles < 1 || (!draw && a.feat_tiles < 1)) return DKF_EINVAL;
    if (draw && (!a.wfrag2 || !a.xfrag2 || !a.bias2 || a.N < 1 || a.S < 1)) return DKF_EINVAL;
    StageTimer timer(stage, stream);
    const int samp_tiles8 = (a.samp_tiles + 7) / 8 * 8;
    if (draw) {
        FragGemmArgs d = a;
        const bool stage_outputs = a.out_mean_dbg || a.out_sd_dbg;
        if (!stage_outputs && a.N % 128 == 0 && a.S % 256 == 0) {
            d.feat_tiles = a.N / 128;
            hipLaunchKernelGGL(frag_draw_whole, dim3(samp_tiles8 * d.feat_tiles), dim3(kThreads), 0, stream, d);
        } else {
            d.feat_tiles = (a.N + 63) / 64;
            const dim3 grid(samp_tiles8 * d.feat_tiles);
            if (stage_outputs) hipLaunchKernelGGL(frag_draw<true>, grid, dim3(kThreads), 0, stream, d);
            else hipLaunchKernelGGL(frag_draw<false>, grid, dim3(kThreads), 0, stream, d);
        }
    } else {
        const dim3 grid(samp_tiles8 * a.feat_tiles);
        if (a.tile == 2) launch_t<2>(a, grid, stream);
        else launch_t<4>(a, grid, stream);
    }
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

}  // namespace dkf
