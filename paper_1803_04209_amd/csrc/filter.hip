// Lagged filtering: fixed-lag window and the two RNN encoders of the inference
// network (Sec. 3.1.3: h_left runs forward over the window, h_right backward,
// both single-layer ReLU cells started from zero).
//
// The input projection W_ih x_t does not depend on where x_t sits in the
// window, so it is computed once per observation (project_observation) and
// kept in a ring; it is stored un-normalised, and the normaliser 1/s is
// applied when the recurrence consumes it (W_ih (x/s) = (W_ih x)/s).
// The recurrences are two chains of L dependent R x R mat-vecs: one workgroup
// per direction, the hidden state in LDS (encode_window).
#include "common.h"

namespace dkf {
namespace {

constexpr int kProjThreads = 256;
constexpr int kProjRowsPerBlock = 4;  // one row per wavefront: R/4 workgroups per direction
constexpr int kChainThreads = 1024;
constexpr float kCoopEmpty = -1.0f;  // "not written yet" in ctx while the multi-workgroup encoder runs (states are >= 0)

// Sum over aligned groups of TPR lanes (TPR a power of two <= 64); every lane of a group gets the
// total.  Up to 16 lanes the partners come by DPP moves (lane ^ 1, lane ^ 2, mirror inside 8, mirror
// inside 16: any pairing across the halves does for a sum), beyond that through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int TPR>
__device__ __forceinline__ float group_sum(float v) {
    if constexpr (TPR >= 2) v += dpp_f<0xB1>(v);
    if constexpr (TPR >= 4) v += dpp_f<0x4E>(v);
    if constexpr (TPR >= 8) v += dpp_f<0x141>(v);
    if constexpr (TPR >= 16) v += dpp_f<0x140>(v);
    if constexpr (TPR >= 32) v += __shfl_xor(v, 16, 64);
    if constexpr (TPR >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// mirror = input (observation + control block; `input` is pinned host memory): one workgroup, every
// read across the bus in flight at once
__global__ __launch_bounds__(1024) void mirror_observation(FilterArgs a) {
    const int n = a.Np + (int)(sizeof(Control) / sizeof(float));
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = threadIdx.x + u * 1024;
        v[u] = i < n ? a.input[i] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = threadIdx.x + u * 1024;
        if (i < n) a.mirror[i] = v[u];
    }
    for (int i = threadIdx.x + 4096; i < n; i += 1024) a.mirror[i] = a.input[i];
}

// proj_dir[slot][r] = sum_j w_ih_dir[r][j] * x[j]      grid: (ceil(R/16), 2)
__global__ __launch_bounds__(kProjThreads) void project_observation(FilterArgs a) {
    const Control ctl = *reinterpret_cast<const Control *>(a.input + a.Np);
    const int dir = blockIdx.y;
    const float *__restrict__ w = dir ? a.w_ih_b : a.w_ih_f;
    float *__restrict__ proj = (dir ? a.proj_b : a.proj_f) + (size_t)ctl.slot * a.R;
    const float *__restrict__ x = a.input;
    if (blockIdx.x == 0 && dir == 0 && a.mirror != a.input) {  // device copy for the kernels that follow
        const int n = a.Np + (int)(sizeof(Control) / sizeof(float));
        for (int i = threadIdx.x; i < n; i += kProjThreads) a.mirror[i] = a.input[i];
    }
    if (a.mark_empty && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        __hip_atomic_store(a.fault, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // this step has not failed yet
        __hip_atomic_store(a.xcd_claims, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.xcd_claims + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (a.mark_empty) {  // the multi-workgroup encoder that follows polls ctx for values >= 0
        const int total = a.L * a.R;
        float *__restrict__ c = dir ? a.ctx_b : a.ctx_f;
        for (int i = blockIdx.x * kProjThreads + threadIdx.x; i < total; i += gridDim.x * kProjThreads)
            c[(size_t)(i / a.R) * a.Rp + i % a.R] = kCoopEmpty;
    }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int N = a.N;
    for (int i = wave; i < kProjRowsPerBlock; i += kProjThreads / 64) {
        const int r = blockIdx.x * kProjRowsPerBlock + i;
        if (r >= a.R) break;
        const float *__restrict__ wr = w + (size_t)r * N;
        float s = 0.f;
        if ((N & 3) == 0) {
            int j = lane * 4;
            for (; j + 768 < N; j += 1024) {  // four independent loads of the matrix row in flight
                float4 wv[4], xv[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    wv[q] = *reinterpret_cast<const float4 *>(wr + j + 256 * q);
                    xv[q] = *reinterpret_cast<const float4 *>(x + j + 256 * q);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) s += wv[q].x * xv[q].x + wv[q].y * xv[q].y + wv[q].z * xv[q].z + wv[q].w * xv[q].w;
            }
            for (; j < N; j += 256) {
                const float4 wv = *reinterpret_cast<const float4 *>(wr + j);
                const float4 xv = *reinterpret_cast<const float4 *>(x + j);
                s += wv.x * xv.x + wv.y * xv.y + wv.z * xv.z + wv.w * xv.w;
            }
        } else {
            for (int j = lane; j < N; j += 64) s += wr[j] * x[j];
        }
        s = wave_sum(s);
        if (lane == 0) proj[r] = s;
    }
}

// ctx_dir[t][r] = h_t,  h_t = relu(proj[slot(t)][r] / s + b[r] + sum_k w_hh[r][k] h_prev[k])
// grid: 2 (direction), block 1024; dynamic LDS: 2 * Rp floats.
__global__ __launch_bounds__(kChainThreads) void encode_window(FilterArgs a) {
    extern __shared__ __align__(16) float lds[];
    const Control ctl = *a.ctl;
    if (ctl.count < a.L) return;  // still warming up: nothing to encode
    const int dir = blockIdx.x;
    const int R = a.R, Rp = a.Rp, L = a.L;
    const float *__restrict__ w = dir ? a.w_hh_b : a.w_hh_f;
    const float *__restrict__ bias = dir ? a.bias_b : a.bias_f;
    const float *__restrict__ proj = dir ? a.proj_b : a.proj_f;
    float *__restrict__ ctx = dir ? a.ctx_b : a.ctx_f;
    float *h_prev = lds, *h_next = lds + Rp;
    for (int r = threadIdx.x; r < Rp; r += kChainThreads) { h_prev[r] = 0.f; h_next[r] = 0.f; }
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    constexpr int kWaves = kChainThreads / 64;
    constexpr int kBatch = 8;  // rows per wavefront pass: 8 x (R/256) float4 loads in flight per lane
    const bool vec = (R & 3) == 0;
    for (int step = 0; step < L; ++step) {
        const int t = dir ? L - 1 - step : step;
        int slot = ctl.oldest + t;
        if (slot >= L) slot -= L;
        const float *__restrict__ p = proj + (size_t)slot * R;
        for (int r0 = wave * kBatch; r0 < R; r0 += kWaves * kBatch) {
            float s[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) s[j] = 0.f;
            if (step > 0) {
                if (vec) {
                    for (int k = lane * 4; k < R; k += 256) {
                        const float4 hv = *reinterpret_cast<const float4 *>(h_prev + k);
                        float4 wv[kBatch];
#pragma unroll
                        for (int j = 0; j < kBatch; ++j) {
                            const int r = r0 + j < R ? r0 + j : R - 1;
                            wv[j] = *reinterpret_cast<const float4 *>(w + (size_t)r * R + k);
                        }
#pragma unroll
                        for (int j = 0; j < kBatch; ++j)
                            s[j] += wv[j].x * hv.x + wv[j].y * hv.y + wv[j].z * hv.z + wv[j].w * hv.w;
                    }
                } else {
                    for (int k = lane; k < R; k += 64) {
                        const float hv = h_prev[k];
#pragma unroll
                        for (int j = 0; j < kBatch; ++j) {
                            const int r = r0 + j < R ? r0 + j : R - 1;
                            s[j] += w[(size_t)r * R + k] * hv;
                        }
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) s[j] = wave_sum(s[j]);
            if (lane == 0) {
#pragma unroll
                for (int j = 0; j < kBatch; ++j) {
                    const int r = r0 + j;
                    if (r < R) {
                        const float v = fmaxf(p[r] * ctl.inv_scale + bias[r] + s[j], 0.f);
                        h_next[r] = v;
                        ctx[(size_t)t * Rp + r] = v;
                    }
                }
            }
        }
        __syncthreads();
        float *tmp = h_prev; h_prev = h_next; h_next = tmp;
    }
}

// Same recurrence with the R x R matrix held in registers for the whole chain:
// 1024 threads, TPR threads per row, each owning KPT consecutive columns
// (TPR * KPT = rows covered = 1024 / TPR).  A step is KPT fused multiply-adds
// per thread against the previous state in LDS, a log2(TPR)-step lane
// reduction and one barrier.
// With `project` the kernel is the first of a decision: it reads the new observation and the
// control block straight from the caller-side staging buffer (pinned host memory: a PCIe round
// trip of about 3 us).  Everything that does not depend on them -- this thread's share of the
// input matrix row, its block of the recurrent matrix, the ring of cached projections -- is
// requested first, so that those loads are in flight during that round trip.
// Dynamic LDS: (L * ROWS + 2 * HSTRIDE + Np + ROWS) floats.
template <int TPR, int KPT>
__global__ __launch_bounds__(kChainThreads) void encode_window_reg(FilterArgs a) {
    constexpr int ROWS = kChainThreads / TPR;
    static_assert(TPR * KPT == ROWS, "square tile");
    constexpr int HSTRIDE = ROWS + (ROWS / KPT) * 4;  // 4 pad floats per column segment: conflict-free b128 reads
    constexpr int kMaxIn = 8;  // float4 of an input-matrix row per thread: N <= 32 TPR (the fused path's limit)
    extern __shared__ __align__(16) float lds[];
    const int dir = blockIdx.x;
    const int R = a.R, L = a.L, N = a.N;
    const float *__restrict__ w = dir ? a.w_hh_b : a.w_hh_f;
    const float *__restrict__ bias = dir ? a.bias_b : a.bias_f;
    float *__restrict__ proj = dir ? a.proj_b : a.proj_f;
    float *__restrict__ ctx = dir ? a.ctx_b : a.ctx_f;
    float *ring = lds;              // [L][ROWS] cached projections by ring slot (zero beyond R)
    float *h0 = lds + L * ROWS;     // two state buffers, padded layout
    float *h1 = h0 + HSTRIDE;
    float *xs = h1 + HSTRIDE;       // [Np] the new observation
    const int tid = threadIdx.x;
    const int row = tid / TPR, seg = tid % TPR, k0 = seg * KPT;

    // 1. the observation and the control block (host memory when `project`)
    const int n_in = a.Np + (int)(sizeof(Control) / sizeof(float));
    float in0 = 0.f, in1 = 0.f;  // elements tid and tid + 1024 (Np + 8 <= 2048 on this path)
    if (a.project) {
        if (tid < n_in) in0 = a.input[tid];
        if (tid + kChainThreads < n_in) in1 = a.input[tid + kChainThreads];
    }
    // 2. device memory: input-matrix row share, recurrent block, projection ring, bias
    const bool vec_in = (N & 3) == 0;
    float4 wi[kMaxIn];
    if (a.project) {
        const float *__restrict__ wrow = (dir ? a.w_ih_b : a.w_ih_f) + (size_t)row * N;
#pragma unroll
        for (int q = 0; q < kMaxIn; ++q) {
            wi[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < R) {
                if (vec_in) {
                    const int j = (q * TPR + seg) * 4;
                    if (j < N) wi[q] = *reinterpret_cast<const float4 *>(wrow + j);
                } else {  // element (4 q + e) * TPR + seg
                    const int j = 4 * q * TPR + seg;
                    if (j < N) wi[q].x = wrow[j];
                    if (j + TPR < N) wi[q].y = wrow[j + TPR];
                    if (j + 2 * TPR < N) wi[q].z = wrow[j + 2 * TPR];
                    if (j + 3 * TPR < N) wi[q].w = wrow[j + 3 * TPR];
                }
            }
        }
    }
    float wreg[KPT];
    if (KPT >= 4 && (R & 3) == 0) {
#pragma unroll
        for (int j = 0; j < KPT; j += 4) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < R && k0 + j < R) v = *reinterpret_cast<const float4 *>(w + (size_t)row * R + k0 + j);
            wreg[j] = v.x; wreg[j + 1 < KPT ? j + 1 : j] = v.y; wreg[j + 2 < KPT ? j + 2 : j] = v.z;
            wreg[j + 3 < KPT ? j + 3 : j] = v.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < KPT; ++j) wreg[j] = (row < R && k0 + j < R) ? w[(size_t)row * R + k0 + j] : 0.f;
    }
    for (int i0 = tid; i0 < L * ROWS; i0 += 4 * kChainThreads) {  // four loads in flight per thread
        float pv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * kChainThreads;
            const int slot = i / ROWS, r = i % ROWS;
            pv[u] = (i < L * ROWS && r < R) ? proj[(size_t)slot * R + r] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * kChainThreads;
            if (i < L * ROWS) ring[i] = pv[u];
        }
    }
    const float my_bias = (seg == 0 && row < R) ? bias[row] : 0.f;
    for (int i = tid; i < 2 * HSTRIDE; i += kChainThreads) h0[i] = 0.f;

    // 3. the observation has arrived: LDS copy, device mirror, control block
    if (a.project) {
        if (tid < a.Np) xs[tid] = in0;
        if (tid + kChainThreads < a.Np) xs[tid + kChainThreads] = in1;
        if (dir == 0 && a.mirror != a.input) {
            if (tid < n_in) a.mirror[tid] = in0;
            if (tid + kChainThreads < n_in) a.mirror[tid + kChainThreads] = in1;
        }
        // control block: floats Np .. Np + 7 of the input, via LDS to every thread
        float *cl = xs + a.Np;
        if (tid >= a.Np && tid < n_in) cl[tid - a.Np] = in0;
        if (tid + kChainThreads >= a.Np && tid + kChainThreads < n_in) cl[tid + kChainThreads - a.Np] = in1;
    }
    __syncthreads();
    Control ctl;
    if (a.project) ctl = *reinterpret_cast<const Control *>(xs + a.Np);
    else ctl = *a.ctl;

    // 4. input projection of the new observation into its ring slot
    if (a.project) {
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < kMaxIn; ++q) {
            if (vec_in) {
                const int j = (q * TPR + seg) * 4;
                if (j < N) {
                    const float4 xv = *reinterpret_cast<const float4 *>(xs + j);
                    s += wi[q].x * xv.x + wi[q].y * xv.y + wi[q].z * xv.z + wi[q].w * xv.w;
                }
            } else {
                const int j = 4 * q * TPR + seg;
                if (j < N) s += wi[q].x * xs[j];
                if (j + TPR < N) s += wi[q].y * xs[j + TPR];
                if (j + 2 * TPR < N) s += wi[q].z * xs[j + 2 * TPR];
                if (j + 3 * TPR < N) s += wi[q].w * xs[j + 3 * TPR];
            }
        }
        s = group_sum<TPR>(s);
        if (seg == 0) {
            ring[ctl.slot * ROWS + row] = row < R ? s : 0.f;
            if (row < R) proj[(size_t)ctl.slot * R + row] = s;
        }
    }
    if (ctl.count < L || !a.encode) return;  // warming up, or only the projection was asked for
    __syncthreads();

    float *h_prev = h0, *h_next = h1;
    for (int step = 0; step < L; ++step) {
        const int t = dir ? L - 1 - step : step;
        int slot = ctl.oldest + t;
        if (slot >= L) slot -= L;
        float s = 0.f;
        const float *hp = h_prev + k0 + seg * 4;
        if (KPT >= 4) {
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;  // four chains instead of one of KPT dependent adds
#pragma unroll
            for (int j = 0; j < KPT; j += 4) {
                const float4 hv = *reinterpret_cast<const float4 *>(hp + j);
                s0 += wreg[j] * hv.x;
                s1 += wreg[j + 1 < KPT ? j + 1 : j] * hv.y;
                s2 += wreg[j + 2 < KPT ? j + 2 : j] * hv.z;
                s3 += wreg[j + 3 < KPT ? j + 3 : j] * hv.w;
            }
            s = (s0 + s1) + (s2 + s3);
        } else {
#pragma unroll
            for (int j = 0; j < KPT; ++j) s += wreg[j] * hp[j];
        }
        s = group_sum<TPR>(s);
        if (seg == 0) {
            const float v = fmaxf(ring[slot * ROWS + row] * ctl.inv_scale + my_bias + s, 0.f);
            h_next[row + (row / KPT) * 4] = v;
            if (row < R) ctx[(size_t)t * a.Rp + row] = v;
        }
        __syncthreads();
        float *tmp = h_prev; h_prev = h_next; h_next = tmp;
    }
}

// The same recurrence for 128 < R <= 256 with four rows per thread: thread (row group, segment) holds
// a 4 x 16 block of the matrix, so a step reads only 16 state values per thread from LDS (a quarter
// of what one row x 64 columns per thread reads: that variant is bound by LDS bandwidth) at the
// price of four 16-lane reductions.  No fused projection: the input terms come from the ring.
// Dynamic LDS: (L * 256 + 2 * 320) floats.
template <bool MERGED>
__device__ __forceinline__ void encode_reg4_body(const FilterArgs &a, int dir) {
    constexpr int ROWS = 256, TPR = 16, KPT = 16, RPT = 4, SEG = KPT + 4, HBUF = TPR * SEG;
    extern __shared__ __align__(16) float lds[];
    const int R = a.R, L = a.L;
    const float *__restrict__ w = dir ? a.w_hh_b : a.w_hh_f;
    const float *__restrict__ bias = dir ? a.bias_b : a.bias_f;
    const float *__restrict__ proj = dir ? a.proj_b : a.proj_f;
    float *__restrict__ ctx = dir ? a.ctx_b : a.ctx_f;
    float *pre = lds;             // [L][ROWS] input term of every step
    float *h = lds + L * ROWS;    // two buffers [TPR][SEG]
    const int tid = threadIdx.x;
    const int rg = tid / TPR, seg = tid % TPR, k0 = seg * KPT;

    // The matrix is the longest transfer of the kernel (256 KiB into one compute unit) and depends
    // on nothing: in the merged kernel it is requested first and the projection workgroups do
    // their work meanwhile.
    float wreg[RPT][KPT];
    auto load_matrix = [&] {
        if (R == ROWS) {  // the whole tile is inside the matrix: plain 16-byte loads
#pragma unroll
            for (int i = 0; i < RPT; ++i)
#pragma unroll
                for (int j = 0; j < KPT; j += 4) {
                    const float4 v = *reinterpret_cast<const float4 *>(w + (size_t)(rg * RPT + i) * ROWS + k0 + j);
                    wreg[i][j] = v.x; wreg[i][j + 1] = v.y; wreg[i][j + 2] = v.z; wreg[i][j + 3] = v.w;
                }
        } else {
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                const int row = rg * RPT + i;
#pragma unroll
                for (int j = 0; j < KPT; ++j) wreg[i][j] = (row < R && k0 + j < R) ? w[(size_t)row * R + k0 + j] : 0.f;
            }
        }
    };
    if (MERGED) load_matrix();
    // merged: the control block comes from where the host put it (later kernels read the mirror
    // that the first projection workgroup writes)
    const Control ctl = MERGED ? *reinterpret_cast<const Control *>(a.input + a.Np) : *a.ctl;
    if (MERGED && tid == 0) __hip_atomic_store(a.fault + 1 + dir, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (ctl.count < L) return;

    // input terms of every step (merged: all but the newest observation's, which is being computed)
    auto input_terms = [&](bool newest) {
        for (int i0 = tid; i0 < L * ROWS; i0 += 4 * kChainThreads) {
            float pv[4], bv[4];
            bool mine[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * kChainThreads;
                const int step = i / ROWS, r = i % ROWS;
                const int t = dir ? L - 1 - step : step;
                int slot = ctl.oldest + t;
                if (slot >= L) slot -= L;
                mine[u] = i < L * ROWS && (!MERGED || (slot == ctl.slot) == newest);
                const bool ok = mine[u] && r < R;
                const float *src = proj + (size_t)slot * R + r;
                // the newest row was written by other workgroups of this launch: read it past the caches
                pv[u] = !ok ? 0.f : (MERGED && newest) ? __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *src;
                bv[u] = ok ? bias[r] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * kChainThreads;
                if (mine[u]) pre[i] = pv[u] * ctl.inv_scale + bv[u];
            }
        }
    };
    input_terms(false);
    if (!MERGED) load_matrix();
    for (int i = tid; i < 2 * HBUF; i += kChainThreads) h[i] = 0.f;
    if (MERGED) {
        // Wait until every projection workgroup has published this step's number (bounded: when the
        // polls run out the direction's fault word is raised and the workgroup leaves; the decision's
        // last kernel and dkf_check report that as DKF_ESTALLED).
        bool arrived = true;
        const int P = (int)gridDim.x - 2;
        if (tid < P) {
            for (int polls = 0;; ++polls) {  // (a limit of zero gives up before the first look)
                if (polls >= a.spin_limit) { arrived = false; break; }
                if (__hip_atomic_load(a.proj_flags + tid, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) == ctl.seq) break;
                __builtin_amdgcn_s_sleep(2);
            }
        }
        if (__syncthreads_or(!arrived)) {
            // no encoding this step: the direction's rows become NaN, so that samples drawn from them
            // cannot pass for a prediction
            if (tid == 0) __hip_atomic_store(a.fault + 1 + dir, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (int i = tid; i < L * R; i += kChainThreads) ctx[(size_t)(i / R) * a.Rp + i % R] = __builtin_nanf("");
            return;
        }
        input_terms(true);
    }
    __syncthreads();

    const int my_row = rg * RPT + (seg & (RPT - 1));  // lanes 0..3 of a row group write one row each
    for (int step = 0; step < L; ++step) {
        const int t = dir ? L - 1 - step : step;
        float s[RPT] = {0.f, 0.f, 0.f, 0.f};
        if (step > 0) {
            const float *hp = h + (step & 1) * HBUF + seg * SEG;
#pragma unroll
            for (int j = 0; j < KPT; j += 4) {
                const float4 hv = *reinterpret_cast<const float4 *>(hp + j);
#pragma unroll
                for (int i = 0; i < RPT; ++i)
                    s[i] = fmaf(wreg[i][j + 3], hv.w, fmaf(wreg[i][j + 2], hv.z, fmaf(wreg[i][j + 1], hv.y, fmaf(wreg[i][j], hv.x, s[i]))));
            }
#pragma unroll
            for (int i = 0; i < RPT; ++i) s[i] = group_sum<TPR>(s[i]);
        }
        float mine = s[0];
#pragma unroll
        for (int i = 1; i < RPT; ++i) mine = (seg & (RPT - 1)) == i ? s[i] : mine;
        if (seg < RPT) {
            const float v = fmaxf(pre[step * ROWS + my_row] + mine, 0.f);
            h[((step + 1) & 1) * HBUF + (my_row / KPT) * SEG + my_row % KPT] = v;
            if (my_row < R) ctx[(size_t)t * a.Rp + my_row] = v;
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(kChainThreads) void encode_window_reg4(FilterArgs a) { encode_reg4_body<false>(a, blockIdx.x); }

// Projection and recurrences of a step in one launch (128 < R <= 256, input matrix too large for the
// two encoder workgroups to read alone).  Workgroups 0 and 1 are the encoders of encode_window_reg4;
// workgroups 2 ... are the projection: 16 rows of one direction each (a wavefront per row), the
// observation read straight from where the host staged it.  The encoders spend their first
// microseconds fetching the recurrent matrix, which is when the projection is computed; a
// projection workgroup publishes the step's number (Control::seq) in its flag word after its rows,
// and an encoder starts the recurrence once every flag shows that number.  Nothing is ever reset:
// the number is different for every step of a model's life.
constexpr int kMergedProjRows = kChainThreads / 64;
__global__ __launch_bounds__(kChainThreads) void encode_window_reg4_merged(FilterArgs a) {
    if (blockIdx.x < 2) {
        encode_reg4_body<true>(a, blockIdx.x);
        return;
    }
    const int pb = blockIdx.x - 2, per_dir = ((int)gridDim.x - 2) / 2;
    const int dir = pb / per_dir;
    const Control ctl = *reinterpret_cast<const Control *>(a.input + a.Np);
    // the observation crosses to this compute unit once (it may sit in host memory), then every
    // wavefront reads it from LDS
    extern __shared__ __align__(16) float xs[];  // [Np]
    {
        const int n = a.Np + (int)(sizeof(Control) / sizeof(float));
        const bool mirror = pb == 0 && a.mirror != a.input;  // device copy for the kernels that follow
        for (int i = threadIdx.x; i < n; i += kChainThreads) {
            const float v = a.input[i];
            if (i < a.Np) xs[i] = v;
            if (mirror) a.mirror[i] = v;
        }
    }
    __syncthreads();
    const float *x = xs;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = (pb % per_dir) * kMergedProjRows + wave;
    const int N = a.N;
    if (r < a.R) {
        const float *__restrict__ wr = (dir ? a.w_ih_b : a.w_ih_f) + (size_t)r * N;
        float s = 0.f;
        if ((N & 3) == 0) {
            for (int j0 = 0; j0 < N; j0 += 1024) {  // up to four 16-byte loads of the row in flight
                float4 wv[4], xv[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = j0 + lane * 4 + 256 * q;
                    const int jc = j < N ? j : 0;
                    wv[q] = *reinterpret_cast<const float4 *>(wr + jc);
                    xv[q] = *reinterpret_cast<const float4 *>(x + jc);
                    if (j >= N) wv[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) s += wv[q].x * xv[q].x + wv[q].y * xv[q].y + wv[q].z * xv[q].z + wv[q].w * xv[q].w;
            }
        } else {
            for (int j = lane; j < N; j += 64) s += wr[j] * x[j];
        }
        s = wave_sum(s);
        if (lane == 0)
            __hip_atomic_store((dir ? a.proj_b : a.proj_f) + (size_t)ctl.slot * a.R + r, s, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(a.proj_flags + pb, ctl.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// Wide encoders (R > 256): the R x R matrix no longer fits one compute unit's registers, so each
// direction is split over P = ceil(R / 64) workgroups of 64 rows, every thread holding KPT
// consecutive columns of one row in registers for the whole chain (16 threads per row).  After
// each step a workgroup publishes its 64 new state values (they are the rows of ctx it owns) and
// reads the full state back: one device-scope exchange of R floats per step instead of streaming
// the matrix from L2 per step.  The data is its own flag: a ReLU output is never negative, the
// projection kernel that precedes this one fills ctx with kCoopEmpty, and thread k polls element
// k of the step's row until it has been written (one memory round trip per step, no counters).
// The wait is bounded: if a value does not arrive within spin_limit polls (kCoopSpinLimit unless
// the host lowered it; it always arrives unless the device is shared with a kernel that never
// ends) the workgroup raises the step's fault word and sets the encodings it owns to NaN with
// device-scope stores (a NaN also ends the wait of every workgroup polling them), and every wave
// still exits.  The decision's last kernel turns a raised fault word into DKF_ESTALLED.
constexpr int kCoopRows = 64;
constexpr int kCoopTpr = kChainThreads / kCoopRows;  // 16 lanes per row = one DPP row

// XCD this wavefront runs on: hardware register XCC_ID (id 20), bits 3:0
__device__ __forceinline__ int xcd_id() { return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 15; }

// Placement of the workgroups (FilterArgs::same_xcd).  The state exchange costs one round trip to
// the level of the memory system at which the workgroups of a direction are coherent: through
// memory (device-scope stores and loads, about 2.3 us per step) when they may sit on different
// XCDs, whose L2 caches are not coherent with each other; through the L2 (stores that stop there,
// about 1.3 us per step) when they all sit on one XCD.  This second form leans on how the hardware
// behaves (L1 write-through, one L2 per XCD), not on the language's memory model, which asks for
// device scope on both sides; the bounded wait turns a failure of that assumption into
// DKF_ESTALLED, never into a hang.  For it a grid of 8 * blocks workgroups is launched; every workgroup reads
// the XCD it landed on, those on XCD 0 take the forward direction and those on XCD 1 the backward
// one, each claiming the next row block of its direction from a counter, and the others leave at
// once.  (The dispatcher deals workgroups to the XCDs in turn, so each XCD receives `blocks` of them;
// filter_xcd_census checks this on the device before the path is enabled.)
template <int KPT>
__global__ __launch_bounds__(kChainThreads) void encode_window_coop(FilterArgs a) {
    constexpr int SEG = KPT + 4;  // 4 pad floats per column segment: conflict-free b128 reads
    constexpr int HBUF = kCoopTpr * SEG;
    extern __shared__ __align__(16) float lds[];
    __shared__ int bail, claim;
    const Control ctl = *a.ctl;
    if (ctl.count < a.L) return;  // still warming up: nothing to encode (uniform over the grid)
    const int tid = threadIdx.x;
    int dir = blockIdx.y, block = blockIdx.x;
    if (a.same_xcd) {
        dir = xcd_id();
        if (dir > 1) return;
        if (tid == 0) claim = __hip_atomic_fetch_add(a.xcd_claims + dir, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        block = claim;
        if (block >= (a.R + kCoopRows - 1) / kCoopRows) return;  // this direction's row blocks are all taken
    }
    const int R = a.R, Rp = a.Rp, L = a.L;
    const float *__restrict__ w = dir ? a.w_hh_b : a.w_hh_f;
    const float *__restrict__ bias = dir ? a.bias_b : a.bias_f;
    const float *__restrict__ proj = dir ? a.proj_b : a.proj_f;
    float *ctx = dir ? a.ctx_b : a.ctx_f;
    float *h = lds;               // two buffers [kCoopTpr][SEG]: previous state by column segment
    float *pre = lds + 2 * HBUF;  // [L][kCoopRows] input term of every step
    const int row_local = tid / kCoopTpr, seg = tid % kCoopTpr;
    const int row = block * kCoopRows + row_local, k0 = seg * KPT;

    float wreg[KPT];
    if (R == kCoopTpr * KPT && (R % kCoopRows) == 0) {  // the whole tile is inside the matrix: plain 16-byte loads
#pragma unroll
        for (int j = 0; j < KPT; j += 4) {
            const float4 v = *reinterpret_cast<const float4 *>(w + (size_t)row * R + k0 + j);
            wreg[j] = v.x; wreg[j + 1] = v.y; wreg[j + 2] = v.z; wreg[j + 3] = v.w;
        }
    } else
#pragma unroll
    for (int j = 0; j < KPT; j += 4) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < R) {
            if ((R & 3) == 0 && k0 + j + 3 < R) {
                v = *reinterpret_cast<const float4 *>(w + (size_t)row * R + k0 + j);
            } else {
                if (k0 + j < R) v.x = w[(size_t)row * R + k0 + j];
                if (k0 + j + 1 < R) v.y = w[(size_t)row * R + k0 + j + 1];
                if (k0 + j + 2 < R) v.z = w[(size_t)row * R + k0 + j + 2];
                if (k0 + j + 3 < R) v.w = w[(size_t)row * R + k0 + j + 3];
            }
        }
        wreg[j] = v.x; wreg[j + 1] = v.y; wreg[j + 2] = v.z; wreg[j + 3] = v.w;
    }
    for (int i0 = tid; i0 < L * kCoopRows; i0 += 4 * kChainThreads) {  // four loads in flight per thread
        float pv[4], bv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * kChainThreads;
            const int step = i / kCoopRows, r = block * kCoopRows + i % kCoopRows;
            const int t = dir ? L - 1 - step : step;
            int slot = ctl.oldest + t;
            if (slot >= L) slot -= L;
            const bool ok = i < L * kCoopRows && r < R;
            pv[u] = ok ? proj[(size_t)slot * R + r] : 0.f;
            bv[u] = ok ? bias[r] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * kChainThreads;
            if (i < L * kCoopRows) pre[i] = pv[u] * ctl.inv_scale + bv[u];
        }
    }
    for (int i = tid; i < 2 * HBUF; i += kChainThreads) h[i] = 0.f;
    if (tid == 0) bail = 0;
    __syncthreads();

    const int my_slot = (tid / KPT) * SEG + tid % KPT;  // where column `tid` of the state sits in a buffer
    for (int step = 0; step < L; ++step) {
        const int t = dir ? L - 1 - step : step;
        float s = 0.f;
        if (step > 0) {
            const float *hp = h + (step & 1) * HBUF + seg * SEG;
#pragma unroll
            for (int j = 0; j < KPT; j += 4) {
                const float4 hv = *reinterpret_cast<const float4 *>(hp + j);
                s += wreg[j] * hv.x + wreg[j + 1] * hv.y + wreg[j + 2] * hv.z + wreg[j + 3] * hv.w;
            }
            s = group_sum<kCoopTpr>(s);
        }
        if (seg == 0 && row < R) {
            const float hv = fmaxf(pre[step * kCoopRows + row_local] + s, 0.f);
            // same XCD: a workgroup-scope store goes through the write-through L1 into the L2 all
            // readers share and is not pushed on to memory first
            if (a.same_xcd) __hip_atomic_store(ctx + (size_t)t * Rp + row, hv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            else __hip_atomic_store(ctx + (size_t)t * Rp + row, hv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (step == L - 1) break;
        // the whole state of this step, written by all workgroups of the direction
        if (tid < R) {
            const float *src = ctx + (size_t)t * Rp + tid;
            // device-scope load either way: it bypasses this compute unit's L1 (a workgroup-scope load
            // may be served from it and never see the value: measured)
            auto poll = [&]() { return __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
            float v = poll();
            int polls = 0;
            bool gave_up = a.spin_limit <= 0;  // a limit of zero counts as a wait that ran out
            while (!gave_up && v < 0.f) {
                if (++polls > a.spin_limit) { gave_up = true; break; }
                __builtin_amdgcn_s_sleep(1);
                v = poll();
            }
            if (gave_up) { bail = 1; v = 0.f; }
            h[((step + 1) & 1) * HBUF + my_slot] = v;
        }
        __syncthreads();
        if (bail) break;
    }
    if (bail) {  // bounded wait ran out: report it, and poison what this workgroup owns
        if (tid == 0) __hip_atomic_store(a.fault, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int i = tid; i < L * kCoopRows; i += kChainThreads) {
            const int r = block * kCoopRows + i % kCoopRows;
            if (r < R)
                __hip_atomic_store(ctx + (size_t)(i / kCoopRows) * Rp + r, __builtin_nanf(""), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

__global__ __launch_bounds__(kChainThreads) void xcd_census(int32_t *counts) {
    if (threadIdx.x == 0) __hip_atomic_fetch_add(counts + xcd_id(), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int KPT>
int launch_encode_coop(const FilterArgs &a, hipStream_t stream) {
    const size_t lds = ((size_t)2 * kCoopTpr * (KPT + 4) + (size_t)a.L * kCoopRows) * sizeof(float);
    if (lds > 60 * 1024) return DKF_EUNSUPPORTED;
    const int blocks = (a.R + kCoopRows - 1) / kCoopRows;
    const dim3 grid = a.same_xcd ? dim3(8 * blocks) : dim3(blocks, 2);
    hipLaunchKernelGGL((encode_window_coop<KPT>), grid, dim3(kChainThreads), lds, stream, a);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

template <int TPR, int KPT>
int launch_encode_reg(const FilterArgs &a, hipStream_t stream) {
    constexpr int ROWS = kChainThreads / TPR;
    constexpr int HSTRIDE = ROWS + (ROWS / KPT) * 4;
    const size_t lds = ((size_t)a.L * ROWS + 2 * HSTRIDE + a.Np + ROWS) * sizeof(float);
    if (lds > 64 * 1024) return DKF_EUNSUPPORTED;
    hipLaunchKernelGGL((encode_window_reg<TPR, KPT>), dim3(2), dim3(kChainThreads), lds, stream, a);
    DKF_HIP_TRY(hipGetLastError());
    return DKF_OK;
}

// dynamic LDS of encode_window_reg for this size, 0 if R is beyond it
size_t reg_encoder_lds(const FilterArgs &a) {
    int rows, kpt;
    if (a.R <= 32) { rows = 32; kpt = 1; }
    else if (a.R <= 64) { rows = 64; kpt = 4; }
    else if (a.R <= 128) { rows = 128; kpt = 16; }
    else if (a.R <= 256) { rows = 256; kpt = 64; }
    else return 0;
    const int hstride = rows + (rows / kpt) * 4;
    return ((size_t)a.L * rows + 2 * hstride + a.Np + rows) * sizeof(float);
}

}  // namespace

int filter_xcd_census(int blocks_per_direction, bool *ok) {
    *ok = false;
    if (blocks_per_direction < 1 || blocks_per_direction > 16) return DKF_OK;
    int32_t *counts = nullptr, host[16] = {};
    DKF_HIP_TRY(hipMalloc(reinterpret_cast<void **>(&counts), sizeof host));
    hipError_t e = hipMemset(counts, 0, sizeof host);
    for (int rep = 0; rep < 3 && e == hipSuccess; ++rep) {  // three launches: the dealing must not depend on where it starts
        hipLaunchKernelGGL(xcd_census, dim3(8 * blocks_per_direction), dim3(kChainThreads), 0, nullptr, counts);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(host, counts, sizeof host, hipMemcpyDeviceToHost);
    (void)hipFree(counts);
    if (e != hipSuccess) { set_last_hip_error(e); return DKF_EHIP; }
    *ok = host[0] == 3 * blocks_per_direction && host[1] == 3 * blocks_per_direction;
    return DKF_OK;
}

int launch_filter(const FilterArgs &args, bool project, bool encode, hipStream_t stream) {
    StageTimer timer(kStageFilter, stream);
    FilterArgs a = args;
    a.encode = encode;
    a.project = false;
    a.mark_empty = false;
    const size_t reg_lds = reg_encoder_lds(a);
    const bool reg_ok = reg_lds != 0 && reg_lds <= 64 * 1024;  // one workgroup per direction, matrix in registers
    // Small encoders: projection and both recurrences in one launch of two workgroups.  A larger
    // input matrix (measured: 256 x 512) is read faster by the many workgroups of the separate
    // projection kernel than by those two.
    const int reg_rows = a.R <= 32 ? 32 : a.R <= 64 ? 64 : a.R <= 128 ? 128 : 256;  // rows the register kernel covers
    const bool fuse = project && reg_ok && (size_t)reg_rows * a.N <= 32768;
    const bool coop = encode && !reg_ok;  // wide encoders or long windows: several workgroups per direction
    // 128 < R <= 256 with a large input matrix: projection and recurrences as one launch
    const bool merged = project && encode && reg_ok && !fuse && a.R > 128 && (a.R + kMergedProjRows - 1) / kMergedProjRows <= 16;
    if (merged) {
        size_t lds = ((size_t)a.L * 256 + 2 * 16 * 20) * sizeof(float);
        if (lds < a.Np * sizeof(float)) lds = a.Np * sizeof(float);  // (the projection workgroups stage the observation)
        const int per_dir = (a.R + kMergedProjRows - 1) / kMergedProjRows;
        hipLaunchKernelGGL(encode_window_reg4_merged, dim3(2 + 2 * per_dir), dim3(kChainThreads), lds, stream, a);
        DKF_HIP_TRY(hipGetLastError());
        return DKF_OK;
    }
    if ((project && !fuse) || coop) {
        if (project && a.input != a.mirror) {  // many workgroups re-read the vector: bring it into HBM first
            hipLaunchKernelGGL(mirror_observation, dim3(1), dim3(kChainThreads), 0, stream, a);
            DKF_HIP_TRY(hipGetLastError());
        }
        a.input = a.mirror;  // (without `project` the observation of the last push is projected again: same result)
        a.mark_empty = coop;
        const dim3 pgrid((a.R + kProjRowsPerBlock - 1) / kProjRowsPerBlock, 2);
        hipLaunchKernelGGL(project_observation, pgrid, dim3(kProjThreads), 0, stream, a);
        DKF_HIP_TRY(hipGetLastError());
    }
    if (fuse || (encode && reg_ok)) {
        a.project = fuse;
        if (a.R <= 32) return launch_encode_reg<32, 1>(a, stream);
        if (a.R <= 64) return launch_encode_reg<16, 4>(a, stream);
        if (a.R <= 128) return launch_encode_reg<8, 16>(a, stream);
        if (!fuse) {  // four rows per thread: a quarter of the LDS reads per step
            const size_t lds = ((size_t)a.L * 256 + 2 * 16 * 20) * sizeof(float);
            hipLaunchKernelGGL(encode_window_reg4, dim3(2), dim3(kChainThreads), lds, stream, a);
            DKF_HIP_TRY(hipGetLastError());
            return DKF_OK;
        }
        return launch_encode_reg<4, 64>(a, stream);
    }
    if (coop) {
        int rc = DKF_EUNSUPPORTED;
        if (a.R <= 256) rc = launch_encode_coop<16>(a, stream);
        else if (a.R <= 512) rc = launch_encode_coop<32>(a, stream);
        else if (a.R <= 768) rc = launch_encode_coop<48>(a, stream);
        else if (a.R <= 1024) rc = launch_encode_coop<64>(a, stream);
        if (rc != DKF_EUNSUPPORTED) return rc;
        // very long windows: the matrix streamed from L2 every step
        hipLaunchKernelGGL(encode_window, dim3(2), dim3(kChainThreads), 2 * a.Rp * sizeof(float), stream, a);
        DKF_HIP_TRY(hipGetLastError());
    }
    return DKF_OK;
}

}  // namespace dkf
