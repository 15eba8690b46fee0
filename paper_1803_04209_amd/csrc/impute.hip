// Censored run-times (Sec. 4.2, "Handling Censored Run-times") on gfx950.
//
// After a cutoff the stragglers are killed, so the server only knows that
// their run-times exceed the censoring time tau.  Each dropped worker gets a
// value from its predictive run-time distribution left-truncated at tau; that
// distribution is represented by the worker's column of the [S][N] sample
// matrix the decision was taken from, so the truncated draw is: among the
// column's entries greater than tau, in sample order, entry number
// floor(u * m), m being their count (tau itself when m = 0).
//
// The matrix is sample-major, so a wavefront reads 64 adjacent workers of one
// row per load.  The rows are cut into segments of kSegRows; one wavefront
// counts one segment for 64 workers (censored_count); then sixteen threads per
// worker add the segment counts, and one of them walks to the segment that
// holds the worker's entry and re-reads only that segment (censored_pick).  Integer and compare work only:
// results do not depend on launch shape or scheduling.
#include "common.h"

namespace dkf {
namespace {

constexpr int kSegRows = 64;

// counts[seg][N]: entries of column w in rows [seg*kSegRows, ...) that exceed tau (0 for observed workers)
__global__ __launch_bounds__(256) void censored_count(const float *__restrict__ samples, int S, int N,
                                                      const uint8_t *__restrict__ censored, float tau, int segs,
                                                      int32_t *__restrict__ counts) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int w = blockIdx.x * 64 + lane;
    const int seg = blockIdx.y * 4 + wave;
    if (seg >= segs || w >= N) return;
    int32_t m = 0;
    if (censored[w]) {
        const int r0 = seg * kSegRows;
        const int r1 = r0 + kSegRows < S ? r0 + kSegRows : S;
        const float *p = samples + (size_t)r0 * N + w;
        int r = r0;
        for (; r + 3 < r1; r += 4) {  // four independent loads in flight
            const float a = p[0], b = p[(size_t)N], c = p[(size_t)2 * N], d = p[(size_t)3 * N];
            m += (a > tau) + (b > tau) + (c > tau) + (d > tau);
            p += (size_t)4 * N;
        }
        for (; r < r1; ++r, p += N) m += *p > tau;
    }
    counts[(size_t)seg * N + w] = m;
}

constexpr int kPickWorkers = 16;  // workers per workgroup
constexpr int kPickChunks = 16;   // threads per worker: each adds a contiguous run of segment counts

// Sixteen threads per worker add the segment counts in sixteen contiguous runs (sixteen loads in
// flight each); one of them then finds the run, the segment and the row that hold draw number
// floor(u * m).  Integer work throughout: the answer does not depend on how the counts are split.
__global__ __launch_bounds__(kPickWorkers *kPickChunks) void censored_pick(
    const float *__restrict__ samples, int S, int N, const float *__restrict__ x_obs,
    const uint8_t *__restrict__ censored, float tau, const float *__restrict__ u, int segs,
    const int32_t *__restrict__ counts, float *__restrict__ x_full, int32_t *__restrict__ n_exceed) {
    __shared__ int32_t run_sum[kPickChunks][kPickWorkers];
    const int wi = threadIdx.x % kPickWorkers, sj = threadIdx.x / kPickWorkers;
    const int w = blockIdx.x * kPickWorkers + wi;
    const bool dropped = w < N && censored[w] != 0;
    const int per = (segs + kPickChunks - 1) / kPickChunks;
    const int s0 = sj * per;
    const int s1 = s0 + per < segs ? s0 + per : segs;
    int32_t sum = 0;
    if (dropped) {
        int s = s0;
        for (; s + 16 <= s1; s += 16) {
            int32_t c[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) c[i] = counts[(size_t)(s + i) * N + w];
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += c[i];
        }
        for (; s < s1; ++s) sum += counts[(size_t)s * N + w];
    }
    run_sum[sj][wi] = sum;
    __syncthreads();
    if (sj != 0 || w >= N) return;
    if (!dropped) {
        x_full[w] = x_obs[w];
        if (n_exceed) n_exceed[w] = -1;
        return;
    }
    int32_t m = 0;
#pragma unroll
    for (int j = 0; j < kPickChunks; ++j) m += run_sum[j][wi];
    if (n_exceed) n_exceed[w] = m;
    if (m == 0) { x_full[w] = tau; return; }
    float uw = u[w];
    uw = uw >= 0.f ? uw : 0.f;  // u is documented to lie in [0, 1); keep a stray value inside the column
    // float x int32 is exact in double, so this is the same integer on any machine
    long pick = (long)floor((double)uw * (double)m);
    if (pick > m - 1) pick = m - 1;
    long before = 0;
    int run = 0;
    for (; run < kPickChunks - 1; ++run) {
        const int32_t c = run_sum[run][wi];
        if (pick < before + c) break;
        before += c;
    }
    // the segment inside that run
    int seg = run * per;
    const int seg_end = seg + per < segs ? seg + per : segs;
    bool found = false;
    while (!found && seg < seg_end) {
        int32_t c[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) c[i] = seg + i < seg_end ? counts[(size_t)(seg + i) * N + w] : 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (!found) {
                if (pick < before + c[i]) { found = true; seg += i; }
                else before += c[i];
            }
        }
        if (!found) seg += 16;
    }
    float out = tau;
    if (found) {
        // the row inside that segment: the whole segment in flight at once, rows past the end read
        // as tau (never counted)
        long seen = before;
        const int r0 = seg * kSegRows;
        float v[kSegRows];
#pragma unroll
        for (int i = 0; i < kSegRows; ++i) v[i] = r0 + i < S ? samples[(size_t)(r0 + i) * N + w] : tau;
        bool done = false;
#pragma unroll
        for (int i = 0; i < kSegRows; ++i) {
            if (!done && v[i] > tau) {
                if (seen == pick) { out = v[i]; done = true; }
                ++seen;
            }
        }
    }
    x_full[w] = out;
}

}  // namespace

size_t impute_workspace_bytes(int S, int N) {
    if (S < 1 || N < 1) return 0;
    const size_t segs = ((size_t)S + kSegRows - 1) / kSegRows;
    return (segs * (size_t)N * sizeof(int32_t) + 255) / 256 * 256;
}

int launch_impute_censored(const float *samples, int S, int N, const float *x_obs, const uint8_t *censored,
                           float tau, const float *u, float *x_full, int32_t *n_exceed, void *workspace,
                           size_t workspace_bytes, hipStream_t stream) {
    if (!samples || !x_obs || !censored || !u || !x_full || !workspace) return DKF_EINVAL;
    if (S < 1 || N < 1 || tau != tau) return DKF_EINVAL;
    if ((size_t)S * (size_t)N > ((size_t)1 << 40)) return DKF_EUNSUPPORTED;
    if (workspace_bytes < impute_workspace_bytes(S, N)) return DKF_EINVAL;
    if ((reinterpret_cast<uintptr_t>(workspace) & 3) != 0) return DKF_EINVAL;
    const int segs = (S + kSegRows - 1) / kSegRows;
    if ((segs + 3) / 4 > 65535) return DKF_EUNSUPPORTED;
    int32_t *counts = static_cast<int32_t *>(workspace);
    const int strips = (N + 63) / 64;
    hipLaunchKernelGGL(censored_count, dim3(strips, (segs + 3) / 4), dim3(256), 0, stream, samples, S, N, censored,
                       tau, segs, counts);
    DKF_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(censored_pick, dim3((N + kPickWorkers - 1) / kPickWorkers), dim3(kPickWorkers * kPickChunks), 0,
                       stream, samples, S, N, x_obs, censored, tau, u, segs,
                       counts, x_full, n_exceed);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

}  // namespace dkf
