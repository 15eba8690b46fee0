// Monte-Carlo order statistics and the cutoff decision on gfx950.
//
// Monte-Carlo estimate of the expected order statistics (Sec. 3.1.1, last
// paragraph), then Omega(c) = c / mean x_(c) and its argmax (Sec. 3).  Two
// kernels:
//   sort_rank_sums : every row of the [S][N] sample matrix is sorted by a
//                    bitonic network held in registers (several keys per lane,
//                    cross-lane exchanges inside one wavefront), and each rank's
//                    values are summed over the rows a lane group visits;
//   rank_means_omega : fixed-order fp64 reduction of the per-block sums, Omega(c) and the
//                    largest maximiser, 64 ranks per workgroup; the workgroup that finishes
//                    last picks the best of the workgroups' candidates.
// Keys are the order-preserving uint32 image of the fp32 bits, so all compares
// are integer min/max; with a permutation requested the worker index rides in
// the low half of a 64-bit key and breaks ties.
#include <mutex>

#include "common.h"
#include "rowsort.h"

namespace dkf {
namespace {


// One lane group sorts one row per iteration; rank sums stay in registers
// across iterations and are combined per block at the end in a fixed order.
// partial: [gridDim.x][E << LG] fp32, indexed by rank.  THREADS: workgroup size (see plan_for).
// PLAIN: the decision's own configuration -- the row fills the network exactly (N = E << LG), the
// rows divide evenly over the lane groups of the grid, values are summed (not reciprocals) and
// neither the sorted rows nor the permutation are stored -- so the loop body has no row or column
// checks at all, and needs fewer registers (its workgroup shape: sort_threads_plain).
template <int E, int LG, bool WITH_PERM, int THREADS, bool PLAIN = false>
__global__ __launch_bounds__(THREADS) void sort_rank_sums(const float *__restrict__ x, int S, int N,
                                                            float *__restrict__ out_sorted,
                                                            int32_t *__restrict__ out_perm,
                                                            float *__restrict__ partial, int rate, float t_floor,
                                                            uint32_t *__restrict__ done_count) {
    using Lay = Layout<E, LG>;
    // the counter of finished workgroups of the kernel that follows starts at zero
    if (done_count && blockIdx.x == 0 && threadIdx.x == 0) *done_count = 0u;
    using T = typename std::conditional<WITH_PERM, uint64_t, uint32_t>::type;
    constexpr int kThreads = THREADS, kWaves = THREADS / 64;
    constexpr int G = 1 << LG;
    constexpr int NPAD = E * G;
    constexpr int kGroupsPerBlock = kThreads / G;
    const int tid = threadIdx.x;
    const int g = tid & (G - 1);
    const int group = tid >> LG;
    const int total_groups = gridDim.x * kGroupsPerBlock;
    const int iters = (S + total_groups - 1) / total_groups;
    const bool vec_ok = (N & 3) == 0;

    float acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;

    for (int it = 0; it < iters; ++it) {
        const int row = (it * gridDim.x + blockIdx.x) * kGroupsPerBlock + group;
        if constexpr (PLAIN && !WITH_PERM) {
            const float *src = x + (size_t)row * NPAD;
            float4 t[E / 4];
#pragma unroll
            for (int q = 0; q < E / 4; ++q) t[q] = *reinterpret_cast<const float4 *>(src + Lay::load_index(g, q * 4));
            uint32_t v[E];
#pragma unroll
            for (int q = 0; q < E / 4; ++q) {
                v[q * 4] = key_of_flat(t[q].x); v[q * 4 + 1] = key_of_flat(t[q].y);
                v[q * 4 + 2] = key_of_flat(t[q].z); v[q * 4 + 3] = key_of_flat(t[q].w);
            }
            sort_in_lane<uint32_t, E>(v);
            merge_up<uint32_t, E, LG, Lay::kLgE + 1>(v, g);
#pragma unroll
            for (int e = 0; e < E; ++e) acc[e] += value_of(v[e]);
            continue;
        }
        const bool valid = row < S;
        const float *src = x + (size_t)(valid ? row : 0) * N;
        T v[E];
        if (vec_ok && N == NPAD) {
            // the row fills the network exactly: every 16-byte load of the row is issued before the
            // first key is formed (an out-of-range group reads row 0 and discards it)
            float4 t[E / 4];
#pragma unroll
            for (int q = 0; q < E / 4; ++q) t[q] = *reinterpret_cast<const float4 *>(src + Lay::load_index(g, q * 4));
#pragma unroll
            for (int q = 0; q < E / 4; ++q) {
                const int i0 = Lay::load_index(g, q * 4);
                const float f[4] = {t[q].x, t[q].y, t[q].z, t[q].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t k = valid ? key_of(f[j]) : kPadKey;
                    if constexpr (WITH_PERM)
                        v[q * 4 + j] = ((uint64_t)k << 32) | (uint32_t)(i0 + j);
                    else
                        v[q * 4 + j] = k;
                }
            }
        } else {
#pragma unroll
        for (int q = 0; q < E / 4; ++q) {
            const int i0 = Lay::load_index(g, q * 4);
            float f[4];
            if (vec_ok && valid && i0 + 3 < N) {
                const float4 t = *reinterpret_cast<const float4 *>(src + i0);
                f[0] = t.x; f[1] = t.y; f[2] = t.z; f[3] = t.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) f[j] = (valid && i0 + j < N) ? src[i0 + j] : 0.f;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool live = valid && i0 + j < N;
                const uint32_t k = live ? key_of(f[j]) : kPadKey;
                if constexpr (WITH_PERM)
                    v[q * 4 + j] = ((uint64_t)k << 32) | (uint32_t)(i0 + j);
                else
                    v[q * 4 + j] = k;
            }
        }
        }

        sort_in_lane<T, E>(v);
        merge_up<T, E, LG, Lay::kLgE + 1>(v, g);

#pragma unroll
        for (int q = 0; q < E / 4; ++q) {
            const int i0 = Lay::rank(g, q * 4);
            float f[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t k;
                if constexpr (WITH_PERM) k = (uint32_t)(v[q * 4 + j] >> 32); else k = v[q * 4 + j];
                f[j] = value_of(k);
                // rank sums of the values, or (rate rule) of their reciprocals, +inf once a value is not above the floor
                if (valid && i0 + j < N) acc[q * 4 + j] += !rate ? f[j] : f[j] > t_floor ? 1.0f / f[j] : INFINITY;
            }
            if (valid && out_sorted) {
                float *dst = out_sorted + (size_t)row * N;
                if (vec_ok && i0 + 3 < N) {
                    *reinterpret_cast<float4 *>(dst + i0) = make_float4(f[0], f[1], f[2], f[3]);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (i0 + j < N) dst[i0 + j] = f[j];
                }
            }
            if constexpr (WITH_PERM) {
                if (valid && out_perm) {
                    int32_t *dst = out_perm + (size_t)row * N;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (i0 + j < N) dst[i0 + j] = (int32_t)(uint32_t)v[q * 4 + j];
                }
            }
        }
    }

    // Combine the groups of this block: first the groups inside a wavefront
    // (lanes g, g+G, ...), then the wavefronts through LDS, 16 keys at a time.
#pragma unroll
    for (int d = G; d < 64; d <<= 1) {
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] += __shfl_xor(acc[e], d, 64);
    }
    constexpr int kChunk = E < 16 ? E : 16;
    __shared__ float red[kWaves][kChunk][G];
    const int wave = tid >> 6;
    const int lane = tid & 63;
    for (int c0 = 0; c0 < E; c0 += kChunk) {
        if (lane < G) {
#pragma unroll
            for (int e = 0; e < E; ++e)
                if (e >= c0 && e < c0 + kChunk) red[wave][e - c0][lane] = acc[e];
        }
        __syncthreads();
        for (int idx = tid; idx < kChunk * G; idx += kThreads) {
            const int e = c0 + idx / G, gg = idx % G;
            float s = red[0][idx / G][gg];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) s += red[w][idx / G][gg];
            const int i = Lay::rank(gg, e);
            partial[(size_t)blockIdx.x * NPAD + i] = s;
        }
        __syncthreads();
    }
}

constexpr int kMeanParts = 16;  // second-level partial sums per rank

// Rank means, Omega and the argmax in one launch (N > 128).  Workgroup b owns ranks 64 b .. 64 b + 63:
// wavefront w adds the per-block sums of rows w, w + 16, ... of those ranks (fp64, four fixed
// chains, sixteen loads in flight), the sixteen wavefront sums of a rank are added in order, and
// the first wavefront turns them into mean and Omega and finds the workgroup's best rank.  Only that
// candidate (16 bytes) crosses workgroups: it is stored with device scope, a counter is advanced
// with release/acquire order, and the workgroup that finds the counter complete reads all
// candidates (at most 64) and writes the decision.  The sort kernel zeroes the counter.
constexpr int kRankThreads = 1024;
struct RankScratch {           // in the caller's workspace after the per-block sums
    double cand_v[64];
    int32_t cand_c[64];
    uint32_t done;
};

__device__ __forceinline__ bool better_rank(double ov, int oc, double mv, int mc) {
    return oc != 0 && (mc == 0 || ov > mv || (ov == mv && oc > mc));
}
// best (Omega, c) of the wavefront; c = 0 marks "none"; equal Omega: the larger c
__device__ __forceinline__ void wave_best(double &bv, int &bc) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const double ov = __shfl_xor(bv, d, 64);
        const int oc = __shfl_xor(bc, d, 64);
        if (better_rank(ov, oc, bv, bc)) { bv = ov; bc = oc; }
    }
}

__global__ __launch_bounds__(kRankThreads) void rank_means_omega(const float *__restrict__ partial, int blocks,
                                                                 int npad, int N, int S, int c_min, int c_max,
                                                                 float t_floor, float *__restrict__ out_mean,
                                                                 float *__restrict__ out_omega,
                                                                 int32_t *__restrict__ out_cstar,
                                                                 const int32_t *ticket, const int32_t *fault,
                                                                 int rate, RankScratch *__restrict__ rs) {
    __shared__ double red[kMeanParts][64];
    const int lane = threadIdx.x & 63, sub = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + lane;
    {
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        if (col < N) {
            const float *src = partial + col;
            int b = sub;
            for (; b + 15 * kMeanParts < blocks; b += 16 * kMeanParts) {
                float v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = src[(size_t)(b + u * kMeanParts) * npad];
#pragma unroll
                for (int u = 0; u < 16; u += 4) {
                    s0 += (double)v[u]; s1 += (double)v[u + 1]; s2 += (double)v[u + 2]; s3 += (double)v[u + 3];
                }
            }
            for (; b + 3 * kMeanParts < blocks; b += 4 * kMeanParts) {
                const float v0 = src[(size_t)b * npad], v1 = src[(size_t)(b + kMeanParts) * npad];
                const float v2 = src[(size_t)(b + 2 * kMeanParts) * npad], v3 = src[(size_t)(b + 3 * kMeanParts) * npad];
                s0 += (double)v0; s1 += (double)v1; s2 += (double)v2; s3 += (double)v3;
            }
            for (; b < blocks; b += kMeanParts) s0 += (double)src[(size_t)b * npad];
        }
        red[sub][lane] = (s0 + s1) + (s2 + s3);
    }
    __syncthreads();
    if (sub != 0) return;
    // one wavefront from here on
    double sum = red[0][lane];
#pragma unroll
    for (int k = 1; k < kMeanParts; ++k) sum += red[k][lane];
    const int c = col + 1;
    double bv = -INFINITY;
    int bc = 0;
    if (col < N) {
        const double m = sum / (double)S;
        double om = -INFINITY;
        if (!rate) {
            if (c >= c_min && c <= c_max && m > (double)t_floor) om = (double)c / m;
        } else if (c >= c_min && c <= c_max && m < INFINITY) {  // m: mean reciprocal; infinite = some sample not above the floor
            om = (double)c * m;
        }
        if (out_mean) out_mean[col] = (float)m;
        if (out_omega) out_omega[col] = (float)om;
        if (om > -INFINITY) { bv = om; bc = c; }
    }
    wave_best(bv, bc);
    uint32_t prev = 0;
    if (lane == 0) {
        __hip_atomic_store(&rs->cand_v[blockIdx.x], bv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&rs->cand_c[blockIdx.x], bc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        prev = __hip_atomic_fetch_add(&rs->done, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    }
    prev = __builtin_amdgcn_readfirstlane(prev);
    if (prev + 1 != gridDim.x) return;
    // the last workgroup: every candidate has been published before the count it saw
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    bv = -INFINITY;
    bc = 0;
    if (lane < (int)gridDim.x) {
        bv = __hip_atomic_load(&rs->cand_v[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bc = __hip_atomic_load(&rs->cand_c[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    wave_best(bv, bc);
    if (lane == 0) {
        const bool none = bc == 0;
        // an earlier kernel of the same decision gave up (the filter's state exchange): the samples
        // behind this c* are not a prediction
        const bool stalled = fault && (__hip_atomic_load(fault, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) |
                                       __hip_atomic_load(fault + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) |
                                       __hip_atomic_load(fault + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) != 0;
        const int cs = none || stalled ? c_max : bc;
        const int st = stalled ? DKF_ESTALLED : none ? CUTOFF_NO_ELIGIBLE : DKF_OK;
        if (ticket) {
            // For a host that watches pinned memory: ticket, status and c* travel as ONE 64-bit word
            // (ticket in the high half, then 16 bits of status and 16 of c*), so whoever sees the
            // ticket has the decision with it and no store has to wait for another (a release
            // store at system scope would first write the whole L2 back).
            const uint64_t word = ((uint64_t)(uint32_t)*ticket << 32) | ((uint64_t)((uint32_t)st & 0xFFFFu) << 16) |
                                  (uint64_t)((uint32_t)cs & 0xFFFFu);
            __hip_atomic_store(reinterpret_cast<uint64_t *>(out_cstar + 2), word, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_SYSTEM);
        }
        out_cstar[0] = cs;
        out_cstar[1] = st;
    }
}

struct SortPlan {
    int e, lg;       // keys per lane, log2(lanes per row)
    int npad;        // e << lg
    int threads;     // workgroup size of sort_rank_sums
    int blocks;      // grid of sort_rank_sums
    bool plain;      // the check-free loop body (and its workgroup shape) applies
};

// workgroup size by padded row width (must match the instantiations in launch_sort_case)
constexpr int sort_threads(int npad) { return npad >= 2048 ? 256 : npad >= 1024 ? 512 : npad >= 512 ? 1024 : 256; }

// Workgroup size of the check-free body.  It needs fewer registers (four wavefronts per SIMD at
// 2048 keys instead of three), so sixteen wavefronts per workgroup fit a compute unit at every
// width up to 2048 and the grid is one or two workgroups per unit: 256-512 partial rows.
constexpr int sort_threads_plain(int npad) { return npad >= 512 && npad <= 2048 ? 1024 : sort_threads(npad); }

SortPlan plan_for(int S, int N, bool want_plain = false) {
    int npad = 8;
    while (npad < N) npad <<= 1;
    SortPlan p;
    // eight keys per lane while a row fits one wavefront (more keys per lane keep more stages inside
    // registers but leave fewer rows in flight: measured no faster at N = 512)
    p.e = npad / 64 > 8 ? npad / 64 : 8;
    int g = npad / p.e;
    p.lg = 0;
    while ((1 << p.lg) < g) ++p.lg;
    p.npad = npad;
    p.plain = false;
    if (want_plain && N == npad && (N & 3) == 0) {
        const int threads = sort_threads_plain(npad);
        // 512 keys with many rows: sixteen keys per lane and two rows per wavefront (an eighth fewer
        // instructions per row: more stages stay inside a lane); with few rows that leaves compute
        // units without work, so then a row keeps a wavefront of its own
        const bool half_wave = npad == 512 && S >= 8192;
        if (half_wave) { p.e = 16; p.lg = 5; g = 32; }
        const int rows = threads / g;
        const int cap = npad >= 2048 ? 256 : npad >= 512 ? 512 : 2048;
        int blocks = (S + rows - 1) / rows;
        if (blocks > cap) blocks = cap;
        if (S % (blocks * rows) == 0) {  // every lane group has a row in every pass
            p.threads = threads;
            p.blocks = blocks;
            p.plain = true;
            return p;
        }
        if (half_wave) { p.e = 8; p.lg = 6; g = 64; }
    }
    p.threads = sort_threads(npad);
    const int rows_per_block = p.threads / g;
    int blocks = (S + rows_per_block - 1) / rows_per_block;
    // Up to eight small workgroups per compute unit (measured best) for narrow rows.  Rows of 512
    // and 1024 keys take larger workgroups and a grid that is resident all at once, each workgroup
    // looping over its share of the rows: fewer partial rows to write and re-read, fewer dispatches
    // (measured 3-5 % faster).  At 2048 keys (three wavefronts per SIMD by registers) larger workgroups
    // were slower; half as many small ones as before halve the partial rows at the same speed.
    const int cap = npad >= 4096 ? 2048 : npad >= 1024 ? 1024 : npad >= 512 ? 512 : 2048;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    p.blocks = blocks;
    return p;
}

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

template <int E, int LG>
void launch_sort(bool perm, bool plain, dim3 grid, hipStream_t st, const float *x, int S, int N, float *srt,
                 int32_t *pm, float *partial, int rate, float t_floor, uint32_t *done) {
    // the same workgroup shape with and without the permutation: the rank sums are added in the
    // same order either way, so the means are bit-identical (the check-free body has a shape of
    // its own: its means agree with the others to rounding)
    constexpr int T = sort_threads(E << LG), TP = T, TPL = sort_threads_plain(E << LG);
    if (perm)
        hipLaunchKernelGGL((sort_rank_sums<E, LG, true, TP>), grid, dim3(TP), 0, st, x, S, N, srt, pm, partial, rate, t_floor, done);
    else if (plain)
        hipLaunchKernelGGL((sort_rank_sums<E, LG, false, TPL, true>), grid, dim3(TPL), 0, st, x, S, N, srt, pm, partial, rate, t_floor, done);
    else
        hipLaunchKernelGGL((sort_rank_sums<E, LG, false, T>), grid, dim3(T), 0, st, x, S, N, srt, pm, partial, rate, t_floor, done);
}

}  // namespace

// where a producer that sorts its own rows leaves their rank sums, and the counter it has to clear
void cutoff_rank_sums_at(void *workspace, int S, int N, float **partial, uint32_t **done) {
    const SortPlan general = plan_for(S, N);
    *partial = static_cast<float *>(workspace);
    RankScratch *rs = reinterpret_cast<RankScratch *>(static_cast<char *>(workspace) +
                                                      align256((size_t)general.blocks * general.npad * sizeof(float)));
    *done = &rs->done;
}
// rows of rank sums the workspace of cutoff_workspace_bytes(S, N) has room for
int cutoff_rank_sum_rows(int S, int N) { return plan_for(S, N).blocks; }

size_t cutoff_workspace_bytes(int S, int N) {
    if (S < 1 || N < 1 || N > 4096) return 0;
    const SortPlan p = plan_for(S, N);
    return align256((size_t)p.blocks * p.npad * sizeof(float)) + align256(sizeof(RankScratch));
}

int launch_cutoff_select(const float *samples, int S, int N, int c_min, int c_max, float t_floor,
                         float *out_sorted, int32_t *out_perm, float *out_mean, float *out_omega,
                         int32_t *out_cstar, void *workspace, size_t workspace_bytes, hipStream_t stream,
                         const int32_t *ticket, const int32_t *fault, int rate, int presorted_blocks) {
    if (!samples || !out_cstar || !workspace) return DKF_EINVAL;
    if (rate && !(t_floor >= 0.f)) return DKF_EINVAL;
    if (S < 1 || N < 1 || c_min < 1 || c_max > N || c_min > c_max) return DKF_EINVAL;
    if (t_floor != t_floor) return DKF_EINVAL;
    if (N > 4096) return DKF_EUNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return DKF_EINVAL;
    if (workspace_bytes < cutoff_workspace_bytes(S, N)) return DKF_EINVAL;
    if ((reinterpret_cast<uintptr_t>(samples) & 15) != 0) return DKF_EINVAL;
    if (out_sorted && (reinterpret_cast<uintptr_t>(out_sorted) & 15) != 0) return DKF_EINVAL;

    const bool perm = out_perm != nullptr;
    const SortPlan general = plan_for(S, N);  // the workspace is laid out for the larger grid
    SortPlan p = plan_for(S, N, !perm && !out_sorted && !rate);
    // presorted_blocks > 0: the producer of the samples has sorted them too and left that many rows of
    // rank sums at the start of the workspace (cutoff_rank_sums_at); only the reduction runs
    if (presorted_blocks > 0) {
        if (perm || out_sorted || rate || N != general.npad || presorted_blocks > general.blocks) return DKF_EINVAL;
        p.blocks = presorted_blocks;
        p.npad = general.npad;
    }
    float *partial = static_cast<float *>(workspace);
    RankScratch *rs = reinterpret_cast<RankScratch *>(static_cast<char *>(workspace) +
                                                      align256((size_t)general.blocks * general.npad * sizeof(float)));
    const dim3 grid(p.blocks);
    if (presorted_blocks <= 0) {
        StageTimer timer(kStageSort, stream);
#define DKF_SORT_CASE(E_, LG_)                                                                    \
    launch_sort<E_, LG_>(perm, p.plain, grid, stream, samples, S, N, out_sorted, out_perm, partial, rate, t_floor, &rs->done); \
    break
        switch (p.npad) {
            case 8: DKF_SORT_CASE(8, 0);
            case 16: DKF_SORT_CASE(8, 1);
            case 32: DKF_SORT_CASE(8, 2);
            case 64: DKF_SORT_CASE(8, 3);
            case 128: DKF_SORT_CASE(8, 4);
            case 256: DKF_SORT_CASE(8, 5);
            case 512: if (p.e == 16) { DKF_SORT_CASE(16, 5); } else { DKF_SORT_CASE(8, 6); }
            case 1024: DKF_SORT_CASE(16, 6);
            case 2048: DKF_SORT_CASE(32, 6);
            case 4096: DKF_SORT_CASE(64, 6);
            default: return DKF_EUNSUPPORTED;
        }
#undef DKF_SORT_CASE
        DKF_HIP_TRY(hipGetLastError());
    }
    {
        StageTimer timer(kStageArgmax, stream);
        hipLaunchKernelGGL(rank_means_omega, dim3((N + 63) / 64), dim3(kRankThreads), 0, stream, partial, p.blocks,
                           p.npad, N, S, c_min, c_max, t_floor, out_mean, out_omega, out_cstar, ticket, fault, rate,
                           rs);
        DKF_HIP_TRY(hipGetLastError());
    }
    return DKF_OK;
}

// ---- the same call for callers that cannot allocate ------------------------------------------
// The per-block rank sums and the second-level sums live in a fixed array of device memory that
// is part of the loaded code object, so the call needs no workspace from anybody.  Every GPU has
// its own copy at its own address; the address is looked up once per device.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)17 << 20;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up on the first call per device)
int static_scratch(void **out) {
    int dev = -1;
    DKF_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return DKF_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        DKF_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255) != 0) return DKF_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DKF_OK;
}
}  // namespace

size_t cutoff_static_scratch_bytes() { return kStaticScratchBytes; }

int launch_cutoff_select_static(const float *samples, int S, int N, int c_min, int c_max, float t_floor,
                                float *out_sorted, int32_t *out_perm, float *out_mean, float *out_omega,
                                int32_t *out_cstar, hipStream_t stream) {
    if (S < 1 || N < 1) return DKF_EINVAL;
    if (N > 4096) return DKF_EUNSUPPORTED;
    if (cutoff_workspace_bytes(S, N) > kStaticScratchBytes) return DKF_EUNSUPPORTED;
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != DKF_OK) return rc;
    // every word of the scratch the kernels read has been written earlier in the same call, so
    // nothing is cleared; what the previous call left behind is never looked at
    return launch_cutoff_select(samples, S, N, c_min, c_max, t_floor, out_sorted, out_perm, out_mean, out_omega,
                                out_cstar, ws, kStaticScratchBytes, stream, nullptr, nullptr, 0);
}

}  // namespace dkf
