// Internal declarations shared by the translation units of libcutoff_dkf.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "cutoff_dkf.h"

namespace dkf {

// ---- error plumbing ---------------------------------------------------------
void set_last_hip_error(hipError_t e);

#define DKF_HIP_TRY(expr)                            \
    do {                                             \
        hipError_t e_ = (expr);                      \
        if (e_ != hipSuccess) {                      \
            ::dkf::set_last_hip_error(e_);           \
            return DKF_EHIP;                         \
        }                                            \
    } while (0)

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// ---- per-kernel timing (HIP events on the launch stream) ----------------------
enum Stage : int {
    kStageFilter = 0,
    kStageGuide = 1,
    kStageEmitHidden = 2,
    kStageEmitMean = 3,
    kStageEmitScaleHidden = 4,
    kStageEmitScaleDraw = 5,
    kStageSort = 6,
    kStageArgmax = 7,
    kStageSampler = 8,  // guide + transition + emission in the register-chained kernel
};

// Records a start event in the constructor and a stop event in the destructor
// when timing is enabled for `stage`; otherwise does nothing.
class StageTimer {
public:
    StageTimer(int stage, hipStream_t stream);
    ~StageTimer();
    StageTimer(const StageTimer &) = delete;
    StageTimer &operator=(const StageTimer &) = delete;

private:
    int slot_;
    int stage_;
    hipStream_t stream_;
};

// ---- device-side control block ------------------------------------------------
// Copied from pinned host memory at the start of every filter step, after the
// N floats of the new observation.  Kernels only read it.
struct Control {
    int32_t slot;       // ring slot the new observation goes to
    int32_t count;      // observations in the window after this push (<= L)
    int32_t oldest;     // ring slot of the oldest observation in the window
    int32_t ticket;     // sequence number of the decision this block belongs to (0: none); echoed next to c*
    float scale;        // normaliser s (0 while warming up)
    float inv_scale;    // 1/s
    uint32_t seed_lo;   // seed of the built-in generator for this step
    uint32_t seed_hi;
    int32_t seq;        // number of this filter step in the life of the model (from 1, never repeated):
                        // what the projection workgroups of the merged filter kernel publish when done
};

// Weights of one dense layer re-tiled as the B operand of the 32x32 matrix instructions,
// 16 bytes per lane and k-group, zero outside [n_out) x [k_in):
//   fp32 (v_mfma_f32_32x32x2_f32):   tiles[nb][kg][lane][4 floats], n = nb*32 + lane%32,
//                                    k = kg*8 + (lane/32)*4 + j;   k_groups = ceil32(k_in) / 8
//   bf16 (v_mfma_f32_32x32x16_bf16): tiles[nb][kg][lane][8 bf16],  k = kg*16 + (lane/32)*8 + j;
//                                    k_groups = ceil64(k_in) / 16
// bias (fp32) is padded with zeros to n_blocks*32.
struct PackedLayer {
    const float *tiles = nullptr;  // raw 16-byte entries
    const float *bias = nullptr;
    int n_out = 0, k_in = 0;
    int n_blocks = 0;  // ceil(n_out / 32)
    int k_groups = 0;
};

// ---- launchers (each enqueues on `stream` and returns a DKF_* code) ------------

// filter.hip
struct FilterArgs {
    const float *input;    // [Np] new observation followed by a Control block; device memory or pinned
                           // host memory (read once by the first kernel of the step)
    float *mirror;         // dev copy of `input` written by that kernel (may equal input)
    const Control *ctl;    // dev: = mirror + Np, what later kernels read
    float *proj_f, *proj_b;  // dev [L][R] raw input projections W_ih x (no bias, not normalised)
    float *ctx_f, *ctx_b;    // dev [L][Rp] encodings, window order, zero padded
    const float *w_ih_f, *w_ih_b;      // dev [R][N]
    const float *w_hh_f, *w_hh_b;      // dev [R][R]
    const float *bias_f, *bias_b;      // dev [R]: b_ih + b_hh
    int N, Np, L, R, Rp;
    int32_t *fault;   // dev int32[3]: [0] set to 1 by the multi-workgroup encoder when its bounded wait ran
                      // out, cleared by the projection kernel that precedes it; [1 + direction] cleared
                      // and, when its wait for the projection runs out, set by that direction's
                      // workgroup of the merged kernel.  Readers take any non-zero word as "stalled".
    int32_t *proj_flags;  // dev int32[32]: Control::seq of the last step whose rows projection workgroup i
                          // of the merged kernel has finished
    int spin_limit;   // polls that wait may take per step (0: give up at the first wait)
    int32_t *xcd_claims;  // dev int32[2]: row blocks handed out so far per direction (same-XCD encoder);
                          // cleared by the projection kernel
    bool same_xcd;    // (multi-workgroup encoder) all workgroups of a direction run on one XCD and hand
                      // their state over through that XCD's L2; false: any placement, through memory
    bool project;  // (register-resident kernel) compute the new observation's projection in-kernel
    bool mark_empty;  // (projection kernel) fill ctx with the multi-workgroup encoder's "not written yet" value
    bool encode;   // run the recurrences (after the projection) when the window is full
};
constexpr int kCoopSpinLimit = 1 << 20;  // default of FilterArgs::spin_limit
// Whether a grid of 8 * blocks_per_direction workgroups of 1024 threads puts at least
// blocks_per_direction of them on XCD 0 and on XCD 1 of the current device (measured by a small
// census kernel; synchronises the device).  *ok is what FilterArgs::same_xcd may be set to.
int filter_xcd_census(int blocks_per_direction, bool *ok);
int launch_filter(const FilterArgs &a, bool project, bool encode, hipStream_t stream);

// guide.hip
struct GuideArgs {
    const Control *ctl;
    const float *ctx_f, *ctx_b;  // [L][Rp]
    PackedLayer comb, mu, sig;   // Z->R (tanh), R->Z, Z->Z (softplus)
    const float *z0;             // [Zp]
    PackedLayer gate1, prop1;    // Z -> H (ReLU)
    PackedLayer gate2, prop2;    // H -> Z (sigmoid / identity)
    PackedLayer lin, tscale;     // Z -> Z (identity / softplus)
    const float *eps_q, *eps_z;  // [L][S][Z], [S][Z] or NULL with the generator
    float *z_last;               // [S][Z] or NULL
    float *z_next_dbg;           // [S][Z] or NULL
    float *z_next;               // [S][Zp] zero padded: input of the emission
    int S, L, Z, Zp, R, Rp, H, Hp;
    bool bf16;  // layers packed as bf16 tiles
};
int launch_guide(const GuideArgs &a, hipStream_t stream);
size_t guide_lds_bytes(int Zp, int Rp, int Hp, bool bf16);
int guide_prepare(int Zp, int Rp, int Hp, bool bf16);  // raises the kernel's LDS limit once per size

// gchain.hip: guide chain + transition in bf16 with the guide's weights in registers
struct GChainArgs {
    const Control *ctl;
    const float *ctx_f, *ctx_b;  // [L][Rp]
    int Rp;
    // 1 KiB weight tiles (32 output features x 16 inputs, bf16): lane l, entry j of tile (ob, ks) is
    // W[32 ob + l % 32][16 ks + 8 (j / 4) + 4 (l / 32) + j % 4].  With Q = gchain_q() tiles of hidden
    // width per wavefront, in this order: comb [w][ob < Q][ks < 4]; mu [w][nb < 2][ks < 2Q] (k-step
    // 2 w Q + ks of the matrix); sig [nb][ks]; gate1, gate2, prop1, prop2 like comb / mu; lin,
    // tscale like sig; emean1 like comb.
    const float *tiles;
    // fp32 biases, zero padded: comb [128 Q], sig [64], gate1 [128 Q], gate2 [64], prop1 [128 Q],
    // prop2 [64], lin [64], tscale [64], emean1 [128 Q]
    const float *bias_table;
    int bias_floats;
    const float *mu_w32, *mu_b32;  // unrounded W_mu [Z][R] and b_mu [Z] for the context's share of the mean
    float *cmu;                    // [L][64] scratch: that share per window position (zero beyond Z)
    const float *z0;               // [64] zero padded
    const float *eps_q, *eps_z;    // [L][S][Z], [S][Z]
    float *z_last, *z_next_dbg;    // [S][Z] or NULL
    float *z_next;                 // [S][Zp] fp32 rows or NULL
    // hidden layer of the emission's mean as bf16 B fragments [ceil(S/32)][h1_k_steps][64 lanes][16 B], or
    // NULL; emit_mean_act: 0 identity, 1 ReLU; h1_k_steps: padded H / 16 of the consumer (at most 8 Q)
    float *h1frag;
    int h1_k_steps, emit_mean_act;
    int S, L, Z, Zp, R, H;
};
int gchain_q(int Z, int R, int H);  // 0: sizes the kernel is not built for
int launch_gchain(const GChainArgs &a, hipStream_t stream);

// egemm.hip: one dense layer on operands in fragment order (1 KiB = 32 rows x 16 k, bf16, the
// k order of GChainArgs::tiles): out^T = epilogue(W x^T + b)
enum FragEpilogue : int {
    kFragIdentity = 0,  // y -> bf16 fragments
    kFragRelu = 1,      // relu(y) -> bf16 fragments
    kFragDraw = 2,      // mean = y2; sd = softplus(y); x = s * (mean + sd * eps) -> [S][N] rows
};
struct FragGemmArgs {
    int tile;            // workgroups of 32 * tile features x 256 samples: 2 or 4
    const float *wfrag;  // [32-feature block][k_steps][64][16 B], feat_tiles * tile blocks
    const float *xfrag;  // [32-sample block][k_steps][64][16 B], samp_tiles * 8 blocks
    const float *bias;   // fp32 per feature, zero padded
    int k_steps, feat_tiles, samp_tiles, epilogue;
    float *out_frag;     // [32-sample block][out_k_steps][64][16 B], out_k_steps = padded features / 16
    int out_k_steps;
    const float *wfrag2, *xfrag2, *bias2;  // kFragDraw: the mean's product, same shapes as wfrag, xfrag, bias
    const Control *ctl;  // kFragDraw: the normaliser
    const float *eps_x;  // [S][N]
    float *out_samples, *out_mean_dbg, *out_sd_dbg;  // [S][N]
    int S, N;
};
int launch_frag_gemm(const FragGemmArgs &a, int stage, hipStream_t stream);

// mlp_gemm.hip
enum Epilogue : int {
    kEpiBias = 0,       // y = acc + b
    kEpiBiasRelu = 1,   // y = relu(acc + b)
    kEpiScaleDraw = 2,  // sd = softplus(acc + b); x = s * (mean + sd * eps)
};
struct GemmArgs {
    const float *A;  // [S][lda] fp32, K columns used (zero padded up to the layer's k_groups*8)
    int lda;
    PackedLayer layer;
    int S;
    int epilogue;
    float *out;  // kEpiBias/kEpiBiasRelu: [S][ldo], all n_blocks*32 columns written (pads = act(0 + 0))
    int ldo;
    // kEpiScaleDraw only:
    const Control *ctl;
    const float *mean;  // [S][ld_mean]
    int ld_mean;
    const float *eps_x;   // [S][N]
    float *out_samples;   // [S][N]
    float *out_mean_dbg;  // [S][N] or NULL
    float *out_sd_dbg;    // [S][N] or NULL
    int N;
    bool bf16;  // layer packed as bf16 tiles: A is rounded to bf16 while it is staged
};
int launch_gemm(const GemmArgs &a, int stage, hipStream_t stream);

// chain.hip: guide + transition + emission in one register-chained kernel
struct ChainArgs {
    const Control *ctl;
    const float *ctx_f, *ctx_b;  // [L][Rp]
    int Rp;
    const float *guide_tiles;    // comb [RB][ZB], mu [ZB][RB], sig [ZB][ZB] tiles of 64 float4
    const float *stream_tiles;   // chunks of chain_chunk_tiles(HB) tiles in consumption order (pack_chain, api.hip)
    int stream_chunks;
    const float *z0;
    // biases, each zero padded to whole 16-blocks, in the order comb, mu, sig, gate1, gate2, prop1,
    // prop2, lin, tscale, emean1, escale1, emean2, escale2
    const float *bias_table;
    const float *eps_q, *eps_z, *eps_x;
    float *mean;  // [S][ld_mean] scratch, also the emission mean for inspection
    int ld_mean;
    float *out_samples;  // [S][N]
    float *sink;         // >= 4 KiB of scratch that masked-off lanes may write to
    float *z_last, *z_next_dbg, *out_mean_dbg, *out_sd_dbg;  // optional
    int S, L, Z, R, H, N, NB;
    int emit_mean_act;
    int split_waves;  // split.hip only: wavefronts per workgroup the streams were packed for (4 or 8)
    // split.hip only, optional (see split_sorts_rows): the workgroup also sorts its sixteen rows and
    // writes their rank sums, [S / 16][N] fp32 by rank, which is what the row-sort kernel would have
    // left for rank_means_omega; *rank_done is that kernel's counter of finished workgroups, cleared here
    float *rank_partial;
    uint32_t *rank_done;
};
// Whether launch_split can sort the rows it draws (ChainArgs::rank_partial): eight wavefronts per
// workgroup, N = 128 or 512 workers (a row fills the sorting network exactly), whole workgroups of
// sixteen samples.
bool split_sorts_rows(int Z, int R, int H, int L, int N, int S, int waves);
// floats of the chained sampler's bias table (widths padded to 16-blocks), itself padded to whole
// KiB: the kernel copies it into LDS a KiB at a time
__host__ __device__ constexpr int chain_bias_floats(int r16, int z16, int h16, int n16) {
    return (r16 + 6 * z16 + 4 * h16 + 2 * n16 + 255) / 256 * 256;
}
// tiles (16 x 16 weights, 1 KiB) per streamed chunk for a hidden width of hb 16-blocks
__host__ __device__ constexpr int chain_chunk_tiles(int hb) { return hb >= 8 ? 32 : 4 * hb; }
bool chain_supported(int Z, int R, int H, int L, int N);
int launch_chain(const ChainArgs &a, hipStream_t stream);

// quad.hip: the same chain with four samples per wavefront (small sample counts).  Same
// arguments; guide_tiles / stream_tiles / bias_table are the quad packing (pack_quad, api.hip):
// 1 KiB tiles of 64 lanes x float4; biases padded to 64 (R, H, N wide) or 16 (Z wide) per block.
constexpr int kQuadChunkTiles = 32;
// Tile positions of the transition layers and of the emission's first layer in the stream.  A
// layer never straddles a chunk; Z -> Z layers take at least four tiles.
struct QuadPlan {
    int gate1, prop1, lin, gate2, prop2, tscale, emean1;
    int head_chunks;  // chunks before the emission's N-wide layers
};
__host__ __device__ constexpr QuadPlan quad_plan(int zq, int hg) {
    const int big = 4 * zq * hg, small = zq * zq < 4 ? 4 : zq * zq;
    const int sizes[7] = {big, big, small, big, big, small, big};
    int at[7] = {0, 0, 0, 0, 0, 0, 0};
    int pos = 0;
    for (int i = 0; i < 7; ++i) {
        if (pos % kQuadChunkTiles + sizes[i] > kQuadChunkTiles) pos = (pos / kQuadChunkTiles + 1) * kQuadChunkTiles;
        at[i] = pos;
        pos += sizes[i];
    }
    return QuadPlan{at[0], at[1], at[2], at[3], at[4], at[5], at[6], (pos + kQuadChunkTiles - 1) / kQuadChunkTiles};
}
bool quad_supported(int Z, int R, int H, int L, int N);
int launch_quad(const ChainArgs &a, hipStream_t stream);

// split.hip: the same chain with sixteen samples per workgroup, every layer split over its four or
// eight wavefronts (ChainArgs::split_waves).  Same arguments; stream_tiles is one stream per wavefront (pack_split, api.hip),
// split_stream_tiles() tiles apart; bias_table is the layout of chain.hip; guide_tiles, stream_chunks
// and mean are not used.
bool split_supported(int Z, int R, int H, int L, int N, int waves);
int split_stream_tiles(int Z, int R, int H, int N, int waves);  // tiles of one wavefront's stream (0: sizes not built)
int launch_split(const ChainArgs &a, hipStream_t stream);

// noise.hip: out[0..n) = standard normals of stream `tensor` (0 eps_q, 1 eps_z, 2 eps_x); the seed
// is read from `ctl` when that is not NULL (captured graphs), else taken from `seed`
int launch_fill_normal3(float *out0, size_t n0, float *out1, size_t n1, float *out2, size_t n2, const Control *ctl,
                        uint64_t seed, hipStream_t stream);  // tensors 0, 1, 2 in one launch

// cutoff_select.hip
int launch_cutoff_select(const float *samples, int S, int N, int c_min, int c_max, float t_floor,
                         float *out_sorted, int32_t *out_perm, float *out_mean, float *out_omega,
                         int32_t *out_cstar, void *workspace, size_t workspace_bytes, hipStream_t stream,
                         const int32_t *ticket = nullptr,  // dev: if set, out_cstar is 16-byte aligned int32[4] and words 2..3 receive
                                                           // one 64-bit word: *ticket << 32 | (status & 0xFFFF) << 16 | c*
                         const int32_t *fault = nullptr,   // dev: if set and non-zero, the status becomes DKF_ESTALLED
                         int rate = 0,  // 1: rank sums of reciprocals, Omega(c) = c * mean_k 1 / x_(c) (needs t_floor >= 0)
                         int presorted_blocks = 0);  // > 0: the rows are sorted already and that many rows of rank sums
                                                     // lie where cutoff_rank_sums_at says; `samples` is not read
size_t cutoff_workspace_bytes(int S, int N);
// For a producer that sorts its own rows (split.hip): where in a workspace of cutoff_workspace_bytes(S, N)
// its rank sums [rows][N] go, the counter it has to clear, and how many rows there is room for.
void cutoff_rank_sums_at(void *workspace, int S, int N, float **partial, uint32_t **done);
int cutoff_rank_sum_rows(int S, int N);
// the same with the workspace in a fixed device array of the library (no allocation anywhere)
int launch_cutoff_select_static(const float *samples, int S, int N, int c_min, int c_max, float t_floor,
                                float *out_sorted, int32_t *out_perm, float *out_mean, float *out_omega,
                                int32_t *out_cstar, hipStream_t stream);
size_t cutoff_static_scratch_bytes();

// impute.hip
int launch_impute_censored(const float *samples, int S, int N, const float *x_obs, const uint8_t *censored,
                           float tau, const float *u, float *x_full, int32_t *n_exceed, void *workspace,
                           size_t workspace_bytes, hipStream_t stream);
size_t impute_workspace_bytes(int S, int N);

// spread.hip
int launch_rank_spread(const float *sorted, int S, int N, const float *mean, float *out_sd, void *workspace,
                       size_t workspace_bytes, hipStream_t stream);
size_t rank_spread_workspace_bytes(int S, int N);

}  // namespace dkf
