// Spread of the predicted order statistics (the +-2 standard-deviation bands
// of Fig. 3) on gfx950.
//
// Input is the row-sorted sample matrix [S][N] and the rank means the cutoff
// rule already produced; output is, per rank c,
//   sd(c) = sqrt( (1/S) sum_k (x_(c),k - mean(c))^2 ).
// Deviations are taken about the known mean, so nothing cancels.
//
// The matrix is read once, row-major.  A workgroup of 16 wavefronts takes 64
// (or, with 16-byte loads, 256) adjacent ranks of kSegRows consecutive rows,
// 16 rows per wavefront with eight loads in flight, adds the 16 wavefront sums
// through LDS in wavefront order and leaves one partial per rank
// (column_sq_dev); the partials of a rank are then added in segment order
// (spread_finish).  Every sum has a fixed order: results do not depend on
// scheduling.
#include "common.h"

namespace dkf {
namespace {

constexpr int kWaves = 16;
constexpr int kWaveRows = 16;
constexpr int kSegRows = kWaves * kWaveRows;  // rows per workgroup and per partial

// partial[seg][N] = sum over the segment's rows of (x - mean)^2, V ranks per lane
template <int V>
__global__ __launch_bounds__(kWaves * 64) void column_sq_dev(const float *__restrict__ sorted, int S, int N,
                                                             const float *__restrict__ mean,
                                                             float *__restrict__ partial) {
    __shared__ float red[kWaves][64 * V];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c0 = (blockIdx.x * 64 + lane) * V;
    const int seg = blockIdx.y;
    const bool live = c0 < N;
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    const int r0 = seg * kSegRows + wave * kWaveRows;
    const int r1 = r0 + kWaveRows < S ? r0 + kWaveRows : S;
    if (live && r0 < S) {
        float m[V];
        if constexpr (V == 4) {
            const float4 t = *reinterpret_cast<const float4 *>(mean + c0);
            m[0] = t.x; m[1] = t.y; m[2] = t.z; m[3] = t.w;
        } else {
            m[0] = mean[c0];
        }
        const float *p = sorted + (size_t)r0 * N + c0;
        int r = r0;
        constexpr int kInFlight = 8;
        for (; r + kInFlight <= r1; r += kInFlight) {
            float x[kInFlight][V];
#pragma unroll
            for (int i = 0; i < kInFlight; ++i) {
                if constexpr (V == 4) {
                    const float4 t = *reinterpret_cast<const float4 *>(p + (size_t)i * N);
                    x[i][0] = t.x; x[i][1] = t.y; x[i][2] = t.z; x[i][3] = t.w;
                } else {
                    x[i][0] = p[(size_t)i * N];
                }
            }
#pragma unroll
            for (int i = 0; i < kInFlight; ++i)
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const float d = x[i][v] - m[v];
                    acc[v] = fmaf(d, d, acc[v]);
                }
            p += (size_t)kInFlight * N;
        }
        for (; r < r1; ++r, p += N)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const float d = p[v] - m[v];
                acc[v] = fmaf(d, d, acc[v]);
            }
    }
#pragma unroll
    for (int v = 0; v < V; ++v) red[wave][lane * V + v] = acc[v];
    __syncthreads();
    if (wave == 0 && live) {
        float sum[V];
#pragma unroll
        for (int v = 0; v < V; ++v) sum[v] = 0.f;
        for (int w = 0; w < kWaves; ++w)
#pragma unroll
            for (int v = 0; v < V; ++v) sum[v] += red[w][lane * V + v];
        float *q = partial + (size_t)seg * N + c0;
        if constexpr (V == 4) {
            *reinterpret_cast<float4 *>(q) = make_float4(sum[0], sum[1], sum[2], sum[3]);
        } else {
            q[0] = sum[0];
        }
    }
}

// four wavefronts per 64 ranks, each adds a contiguous quarter of the partials; quarters added in order
__global__ __launch_bounds__(256) void spread_finish(const float *__restrict__ partial, int S, int N, int segs,
                                                     float *__restrict__ out_sd) {
    __shared__ float red[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;
    const int per = (segs + 3) / 4;
    const int s0 = wave * per;
    const int s1 = s0 + per < segs ? s0 + per : segs;
    float sum = 0.f;
    if (c < N) {
        int s = s0;
        for (; s + 8 <= s1; s += 8) {
            float t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) t[i] = partial[(size_t)(s + i) * N + c];
#pragma unroll
            for (int i = 0; i < 8; ++i) sum += t[i];
        }
        for (; s < s1; ++s) sum += partial[(size_t)s * N + c];
    }
    red[wave][lane] = sum;
    __syncthreads();
    if (wave == 0 && c < N) {
        const float total = ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
        out_sd[c] = sqrtf(total / (float)S);
    }
}

}  // namespace

size_t rank_spread_workspace_bytes(int S, int N) {
    if (S < 1 || N < 1) return 0;
    const size_t segs = ((size_t)S + kSegRows - 1) / kSegRows;
    return (segs * (size_t)N * sizeof(float) + 255) / 256 * 256;
}

int launch_rank_spread(const float *sorted, int S, int N, const float *mean, float *out_sd, void *workspace,
                       size_t workspace_bytes, hipStream_t stream) {
    if (!sorted || !mean || !out_sd || !workspace) return DKF_EINVAL;
    if (S < 1 || N < 1) return DKF_EINVAL;
    if ((size_t)S * (size_t)N > ((size_t)1 << 40)) return DKF_EUNSUPPORTED;
    if (workspace_bytes < rank_spread_workspace_bytes(S, N)) return DKF_EINVAL;
    const int segs = (S + kSegRows - 1) / kSegRows;
    if (segs > 65535) return DKF_EUNSUPPORTED;
    float *partial = static_cast<float *>(workspace);
    const uintptr_t bits = reinterpret_cast<uintptr_t>(sorted) | reinterpret_cast<uintptr_t>(mean) |
                           reinterpret_cast<uintptr_t>(workspace);
    if ((bits & 3) != 0) return DKF_EINVAL;
    const bool wide = N % 4 == 0 && (bits & 15) == 0;
    if (wide) {
        hipLaunchKernelGGL(column_sq_dev<4>, dim3((N / 4 + 63) / 64, segs), dim3(kWaves * 64), 0, stream, sorted, S, N,
                           mean, partial);
    } else {
        hipLaunchKernelGGL(column_sq_dev<1>, dim3((N + 63) / 64, segs), dim3(kWaves * 64), 0, stream, sorted, S, N, mean,
                           partial);
    }
    DKF_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(spread_finish, dim3((N + 63) / 64), dim3(256), 0, stream, partial, S, N, segs, out_sd);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

}  // namespace dkf
