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
// counts one segment for 64 workers (censored_count), then one lane per
// worker walks the segment counts to the segment that holds its entry and
// re-reads only that segment (censored_pick).  Integer and compare work only:
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

__global__ __launch_bounds__(64) void censored_pick(const float *__restrict__ samples, int S, int N,
                                                    const float *__restrict__ x_obs,
                                                    const uint8_t *__restrict__ censored, float tau,
                                                    const float *__restrict__ u, int segs,
                                                    const int32_t *__restrict__ counts, float *__restrict__ x_full,
                                                    int32_t *__restrict__ n_exceed) {
    const int w = blockIdx.x * 64 + threadIdx.x;
    if (w >= N) return;
    if (!censored[w]) {
        x_full[w] = x_obs[w];
        if (n_exceed) n_exceed[w] = -1;
        return;
    }
    int32_t m = 0;
    for (int s = 0; s < segs; ++s) m += counts[(size_t)s * N + w];
    if (n_exceed) n_exceed[w] = m;
    if (m == 0) { x_full[w] = tau; return; }
    float uw = u[w];
    uw = uw >= 0.f ? uw : 0.f;  // u is documented to lie in [0, 1); keep a stray value inside the column
    // float x int32 is exact in double, so this is the same integer on any machine
    long pick = (long)floor((double)uw * (double)m);
    if (pick > m - 1) pick = m - 1;
    int seg = 0;
    long before = 0;
    for (;; ++seg) {
        const int32_t c = counts[(size_t)seg * N + w];
        if (pick < before + c) break;
        before += c;
    }
    long seen = before;
    const int r0 = seg * kSegRows;
    const int r1 = r0 + kSegRows < S ? r0 + kSegRows : S;
    float out = tau;
    for (int r = r0; r < r1; ++r) {
        const float v = samples[(size_t)r * N + w];
        if (v > tau) {
            if (seen == pick) { out = v; break; }
            ++seen;
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
    hipLaunchKernelGGL(censored_pick, dim3(strips), dim3(64), 0, stream, samples, S, N, x_obs, censored, tau, u, segs,
                       counts, x_full, n_exceed);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

}  // namespace dkf
