/*
 * cutoff_dkf.h -- C ABI of the MI355X (gfx950) Cutoff-SGD run-time predictor.
 *
 * The library implements the parameter server's predict_cutoff call of
 * Teng & Wood, "High Throughput Synchronous Distributed Stochastic Gradient
 * Descent" (Alg. 1, server loop): from the last L observed N-worker run-time
 * vectors it draws S joint predictions of the next run-time vector from the
 * learned deep generative dynamical model (Sec. 3.1.2-3.1.3) and returns the
 * cutoff c* = argmax_c c / E[x_(c)] (Sec. 3; Monte-Carlo order statistics,
 * Sec. 3.1.1, last paragraph).
 *
 * Conventions
 *   - Every function returns an int: 0 = DKF_OK, > 0 = informational status,
 *     < 0 = error.  Nothing throws, aborts or prints.
 *   - "host" pointers are ordinary process memory, "dev" pointers are HIP
 *     device memory on the current device.  The caller owns every buffer it
 *     passes in and must keep it alive until the work queued on `stream` has
 *     finished; the library never frees or reallocates caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Unless stated otherwise calls only enqueue work and return; results are
 *     valid once the caller has synchronised the stream.
 *   - Matrices are row-major; sample tensors are sample-major ([S][.]), so one
 *     sampled N-vector is contiguous.
 *   - Calls on one dkf_model must not overlap in time (one stream at a time).
 */
#ifndef CUTOFF_DKF_H
#define CUTOFF_DKF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status / error codes */
#define DKF_OK 0
#define DKF_WARMUP 1             /* fewer than L observations so far: no prediction possible, use c = N */
#define CUTOFF_NO_ELIGIBLE 2     /* no cutoff passed the floor; c* was set to c_max */
#define DKF_EINVAL (-1)          /* bad dimension, NULL pointer, c_min > c_max, S < 1 ... */
#define DKF_ENOTREADY (-2)       /* sampling requested before L observations were pushed */
#define DKF_EBADOBS (-3)         /* an observed run-time was non-finite or <= 0 */
#define DKF_EHIP (-4)            /* a HIP runtime call failed; see dkf_last_hip_error() */
#define DKF_ENOMEM (-5)          /* host or device allocation failed */
#define DKF_EBLOB (-6)           /* weight blob header/size does not match the configuration */
#define DKF_EUNSUPPORTED (-7)    /* a size beyond what the kernels are built for (see each call) */
#define DKF_ESTALLED (-8)        /* the filter's workgroups stopped waiting for each other: no valid encoding, no decision */

#define DKF_DTYPE_F32 0          /* MLP GEMMs in fp32 */
#define DKF_DTYPE_BF16 1         /* MLP GEMM inputs rounded to bf16, fp32 accumulate */

typedef struct dkf_model dkf_model; /* opaque: device weights, fixed-lag window, workspace */

typedef struct {
    int32_t n_workers;     /* N  */
    int32_t lag;           /* L: window length (the paper's l; l = 20 in its experiments, Sec. 4) */
    int32_t z_dim;         /* Z: latent dimension */
    int32_t hidden;        /* H: hidden width of every two-layer MLP (transition, emission) */
    int32_t rnn_dim;       /* R: width of the two RNN encoders = width of h_out */
    int32_t mlp_dtype;     /* DKF_DTYPE_F32 or DKF_DTYPE_BF16 */
    int32_t emit_mean_act; /* hidden nonlinearity of the emission mean I: 0 = identity (as printed, Sec. 3.1.3), 1 = ReLU */
    int32_t max_samples;   /* largest S that will be requested; sizes the workspace */
} dkf_config;

/* Optional per-stage outputs of dkf_sample_runtimes (all dev, any may be NULL). */
typedef struct {
    float *ctx;       /* [L][R]  h_left + h_right per window position (Sec. 3.1.3, guide) */
    float *z_last;    /* [S][Z]  z_T, last step of each guide trajectory */
    float *z_next;    /* [S][Z]  z_{T+1} drawn from the gated transition */
    float *emit_mean; /* [S][N]  I(z_{T+1}), in units of the normaliser */
    float *emit_sd;   /* [S][N]  J(z_{T+1}), in units of the normaliser */
} dkf_stage_outputs;

const char *dkf_strerror(int code);
int dkf_last_hip_error(void); /* hipError_t of the most recent DKF_EHIP on this thread */

/* Number of bytes a weight blob must have for `cfg`.  Blob format (host,
 * little endian): int32[8] {0x57464B44 'DKFW', 1, N, L, Z, H, R, 0} followed
 * by fp32 tensors, each matrix [out][in] row-major so that a layer is
 * W x + b (MLP_n / RNN of Sec. 3.1.3), in this order:
 *   RNN forward : w_ih[R][N] b_ih[R] w_hh[R][R] b_hh[R];  RNN backward: same
 *   guide       : comb_w[R][Z] comb_b[R]  mu_w[Z][R] mu_b[Z]  sig_w[Z][Z] sig_b[Z]  z0[Z]
 *   transition  : gate1_w[H][Z] gate1_b[H] gate2_w[Z][H] gate2_b[Z]
 *                 prop1_w[H][Z] prop1_b[H] prop2_w[Z][H] prop2_b[Z]
 *                 lin_w[Z][Z] lin_b[Z]  tscale_w[Z][Z] tscale_b[Z]
 *   emission    : emean1_w[H][Z] emean1_b[H] emean2_w[N][H] emean2_b[N]
 *                 escale1_w[H][N] escale1_b[H] escale2_w[N][H] escale2_b[N]   */
size_t dkf_blob_bytes(const dkf_config *cfg);

/* Create a model: copies the blob to the device (re-tiled for the matrix
 * cores, converted to bf16 where cfg->mlp_dtype asks for it), allocates the
 * window and a workspace for cfg->max_samples samples.  `blob` is host memory
 * and may be released on return (the call synchronises `stream`).
 * Limits: 1 <= N <= 4096; Z, H, R <= 1024; L <= 256; and one workgroup's
 * share of the guide chain must fit the 160 KB of LDS: with Zp, Hp, Rp the
 * sizes rounded up to a multiple of 32 (fp32) or 64 (bf16),
 *   fp32: 648 Zp + 132 max(Rp, Hp) <= 147456   (Z = 64 with H, R <= 800; Z = H = R <= 160)
 *   bf16: 516 Zp +  66 max(Rp, Hp) <= 147456   (Z = 64 with H, R <= 1024; Z = H = R <= 192)
 * Anything beyond returns DKF_EUNSUPPORTED; there is no slower fall-back.
 * Errors: DKF_EINVAL, DKF_EBLOB, DKF_EUNSUPPORTED, DKF_ENOMEM, DKF_EHIP. */
int dkf_load_weights(const dkf_config *cfg, const void *blob, size_t blob_bytes, void *stream, dkf_model **out);

int dkf_free(dkf_model *m);  /* synchronises the device, releases everything the model owns */
int dkf_reset(dkf_model *m); /* forget the window and the normaliser (next L steps warm up again) */

/* Lagged filtering (Sec. 3.1.2-3.1.3): append one observed run-time vector
 * x_obs[N] (host, seconds, every entry finite and > 0) to the fixed-lag
 * window and re-encode the window with the forward and backward ReLU RNNs of
 * the inference network.  Observations are divided by twice the mean of the
 * first complete window (end of Sec. 3.1.3); that scalar is fixed when the
 * L-th vector arrives.  x_obs is copied before the call returns.
 * Returns DKF_WARMUP until L vectors have been pushed, then DKF_OK.
 * Errors: DKF_EINVAL, DKF_EBADOBS (window unchanged), DKF_EHIP. */
int dkf_filter_step(dkf_model *m, const float *x_obs, void *stream);

/* Posterior-predictive sampling (Sec. 3.1.3, last display): S independent
 * guide trajectories z_1..z_L ~ q(z_t | z_{t-1}, x), one gated-transition
 * draw z_{T+1} ~ N(G(z_T), H(z_T)) and one emission draw
 * x_{T+1} ~ N(I(z_{T+1}), J(z_{T+1})) each, returned in seconds.
 *   eps_q [L][S][Z], eps_z [S][Z], eps_x [S][N]: dev, fp32 standard normals
 *     that drive the three reparameterised draws.  If all three are NULL the
 *     library draws them itself: element i of tensor t (0 eps_q, 1 eps_z,
 *     2 eps_x) is output i mod 4 of Box-Muller on Philox4x32-10 with counter
 *     (i/4 low, i/4 high, t, 0) and key (seed low, seed high), the uniforms
 *     being u1 = ((w >> 8) + 1) / 2^24 and u2 = (w >> 8) / 2^24.
 *   out_samples [S][N] dev, caller-owned; `stages` may be NULL.
 * Errors: DKF_EINVAL (S < 1, S > max_samples, some but not all eps NULL),
 * DKF_ENOTREADY (window not full), DKF_EHIP. */
int dkf_sample_runtimes(dkf_model *m, int32_t S, const float *eps_q, const float *eps_z, const float *eps_x,
                        uint64_t seed, float *out_samples, const dkf_stage_outputs *stages, void *stream);

/* Monte-Carlo order statistics and the cutoff (Sec. 3.1.1 last paragraph;
 * Sec. 3, definition of Omega): sort each of the S rows of `samples` [S][N]
 * (dev) ascending, average every rank over the rows, evaluate
 * Omega(c) = c / mean x_(c) for c in [c_min, c_max] whose mean exceeds
 * t_floor, and write the maximiser (1-based; ties go to the largest c).
 * Model-free: works on any sample matrix.
 *   Order of equal keys: -0 before +0, NaN last, then lower worker index.
 *   out_sorted [S][N] fp32, out_perm [S][N] int32 (0-based worker per rank),
 *   out_mean [N], out_omega [N] (-inf where ineligible): dev, optional (NULL).
 *   out_cstar: dev int32[2] = {c*, status}; status is DKF_OK or
 *     CUTOFF_NO_ELIGIBLE (then c* = c_max).  Required.
 *   workspace: dev, at least cutoff_select_workspace(S, N) bytes, 256-byte
 *     aligned; contents are scratch.
 * Limits: 1 <= N <= 4096, S >= 1.
 * Errors: DKF_EINVAL, DKF_EUNSUPPORTED, DKF_EHIP. */
int cutoff_select(const float *samples, int32_t S, int32_t N, int32_t c_min, int32_t c_max, float t_floor,
                  float *out_sorted, int32_t *out_perm, float *out_mean, float *out_omega, int32_t *out_cstar,
                  void *workspace, size_t workspace_bytes, void *stream);
size_t cutoff_select_workspace(int32_t S, int32_t N);

/* The cutoff under the other reading of "expected gradients per second"
 * (Sec. 3, definition of Omega): the expectation of the ratio,
 * Omega(c) = E[c / x_(c)], estimated by the mean over the sampled rows of
 * c / x_(c), where cutoff_select takes the ratio c / E[x_(c)].  A rank is
 * eligible only if every sampled value of it exceeds t_floor, which must be
 * >= 0 (the Gaussian emission of Sec. 3.1.3 also draws non-positive times,
 * whose reciprocal means nothing); by Jensen's inequality this Omega is never
 * below cutoff_select's.  Arguments, order of equal keys, workspace, bounds,
 * ties, status and errors as for cutoff_select, except:
 *   out_rate [N] (dev, optional): mean over the rows of 1 / x_(c), +inf where
 *     some row's value is <= t_floor (or the fp32 sum overflows);
 *   out_omega [N]: c * out_rate, -inf where ineligible;
 *   t_floor < 0 or NaN: DKF_EINVAL. */
int cutoff_select_rate(const float *samples, int32_t S, int32_t N, int32_t c_min, int32_t c_max, float t_floor,
                       float *out_sorted, int32_t *out_perm, float *out_rate, float *out_omega, int32_t *out_cstar,
                       void *workspace, size_t workspace_bytes, void *stream);

/* cutoff_select for callers that cannot allocate device memory or hand over a
 * workspace: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and error codes as
 * cutoff_select, without the workspace: the per-block rank sums live in a
 * fixed array of cutoff_select_static_max_workspace() bytes (17 MiB) of device
 * memory that belongs to the library; each GPU the library runs on holds its
 * own copy until the process ends.  The call allocates and frees nothing (its
 * first call on a device looks the array's address up, so make that call
 * outside a capture).
 *   Limit: cutoff_select_workspace(S, N) <= cutoff_select_static_max_workspace()
 *   (every N <= 2048 with any S; N <= 4096 with S <= 4096), otherwise
 *   DKF_EUNSUPPORTED and nothing is launched.
 *   All calls on one GPU share the array: calls that overlap in time on one
 *   GPU (different streams, different threads) race and give wrong results;
 *   calls ordered on one stream are safe.  The array keeps the last call's
 *   contents; nothing in it needs clearing between calls. */
int cutoff_select_static(const float *samples, int32_t S, int32_t N, int32_t c_min, int32_t c_max, float t_floor,
                         float *out_sorted, int32_t *out_perm, float *out_mean, float *out_omega,
                         int32_t *out_cstar, void *stream);
size_t cutoff_select_static_max_workspace(void);

/* Spread of the predicted order statistics (Fig. 3 draws every predicted
 * order statistic with a band of two standard deviations): for each rank c,
 *   out_sd[c-1] = sqrt( (1/S) sum_k (sorted[k][c-1] - mean[c-1])^2 ).
 *   sorted [S][N] dev fp32: rows ascending, the out_sorted of cutoff_select;
 *   mean [N] dev fp32: the out_mean of the same call;  out_sd [N] dev fp32.
 *   (Nothing here depends on the rows being sorted: it is the spread of every
 *   column about the given centre, divisor S.)
 *   workspace: dev, at least cutoff_rank_spread_workspace(S, N) bytes, 4-byte
 *     aligned; contents are scratch.  All buffers caller-owned.
 * Sums run in a fixed order: the result does not depend on scheduling.
 * Errors: DKF_EINVAL (null or misaligned pointer, S < 1, N < 1, workspace too
 * small), DKF_EUNSUPPORTED (S * N > 2^40), DKF_EHIP. */
int cutoff_rank_spread(const float *sorted, int32_t S, int32_t N, const float *mean, float *out_sd, void *workspace,
                       size_t workspace_bytes, void *stream);
size_t cutoff_rank_spread_workspace(int32_t S, int32_t N);

/* One whole decision (the predict_cutoff call of Alg. 1): filter_step,
 * sample_runtimes with S samples and cutoff_select over c in [1, N] with floor
 * 0, replayed from a captured HIP graph after the first call with a given S.
 * Noise comes from the caller's tensors (eps_* as in dkf_sample_runtimes, read
 * at every call from the same addresses) or, if they are NULL, from `seed`.
 * Blocks until the decision has arrived and writes c* to *cstar_host.  (The
 * last kernel of the graph stores the decision and a per-call ticket, as one
 * 64-bit word, in pinned host memory, which the call watches; every kernel of the decision has
 * finished by then, but the stream may report busy for a few microseconds
 * more.  If the ticket does not arrive the stream is synchronised instead.)
 * Returns DKF_OK, DKF_WARMUP (then *cstar_host = N), CUTOFF_NO_ELIGIBLE, or
 * an error (DKF_ESTALLED: see dkf_check; *cstar_host = N then).  DKF_EINVAL and DKF_EBADOBS leave the model untouched; after any
 * other error the observation has already entered the window but the
 * decision is lost: restore the window (dkf_set_state) or start over
 * (dkf_reset) before deciding again. */
int dkf_decide(dkf_model *m, const float *x_obs, int32_t S, const float *eps_q, const float *eps_z,
               const float *eps_x, uint64_t seed, int32_t *cstar_host, void *stream);

/* Sequential online replay: the server loop of Alg. 1 with the model in it.
 * For t = 0 .. T-1 row t of trace_host ([T][N], host memory, seconds) is pushed
 * and decided on exactly as by dkf_decide(m, trace_host + t N, S, eps_*, seed + t,
 * ...); the filtering state is carried from step to step.  Per-step results go to
 * host arrays of T entries, each of which may be NULL: cstar_host (c* of the
 * step; N while warming up), status_host (what dkf_decide returned: DKF_OK,
 * DKF_WARMUP, CUTOFF_NO_ELIGIBLE or DKF_ESTALLED) and latency_us_host (wall time
 * of the step on the calling thread, from the observation in hand to c* in
 * hand).  Stops at the first step whose dkf_decide returns another error and
 * returns that code (entries from that step on are not written); else DKF_OK.
 * DKF_EINVAL for a NULL model or trace or T < 1. */
int dkf_decide_trace(dkf_model *m, const float *trace_host, int32_t T, int32_t S, const float *eps_q,
                     const float *eps_z, const float *eps_x, uint64_t seed, int32_t *cstar_host,
                     int32_t *status_host, float *latency_us_host, void *stream);

/* Failure detection for filters whose workgroups wait for each other inside a
 * launch: wide encoders (R > 256), whose recurrence is split over several
 * workgroups that hand their part of the state to each other through memory
 * every step, and encoders of 129-256 units with more than 128 workers, whose
 * two workgroups wait for the input projection computed by other workgroups of
 * the same launch.  A workgroup waits a bounded
 * number of polls; if that runs out (it cannot unless something else holds the
 * device for seconds) it raises a fault word, fills its encodings with NaN and
 * exits.  dkf_decide then returns DKF_ESTALLED instead of a cutoff (never
 * CUTOFF_NO_ELIGIBLE).  For the separate calls, dkf_check synchronises `stream`
 * and returns DKF_ESTALLED if the most recent dkf_filter_step on the model gave
 * up (DKF_OK otherwise): samples drawn from that window are NaN.  The fault is
 * cleared by the next filter step; the window itself is intact.
 * dkf_set_exchange_spin_limit sets the number of polls (default 2^20; 0 makes
 * every wait count as having run out, which is how the tests reach this path
 * with all workgroups still exiting normally).  Host calls. */
int dkf_check(dkf_model *m, void *stream);
int dkf_set_exchange_spin_limit(dkf_model *m, int32_t polls);

/* Device pointer to the [S][N] samples of the last dkf_decide (valid until the
 * next call on the model). */
const float *dkf_decide_samples(const dkf_model *m);

/* Censored run-times (Sec. 4.2): once the server has stopped waiting at time
 * tau (the c-th arrival) the workers still running are killed and their
 * run-times are unknown, but the filter needs a full vector.  Every dropped
 * worker w gets a draw from its predictive run-time distribution
 * left-truncated at tau.  That distribution is represented by column w of
 * the [S][N] sample matrix the decision was taken from (dkf_decide_samples, or
 * the output of dkf_sample_runtimes), so the draw is: of the m entries of
 * column w that are > tau, taken in sample order, entry floor(u[w] * m);
 * tau itself when m = 0.  Observed workers keep x_obs[w].
 *   samples [S][N], x_obs [N] (entries of dropped workers are ignored),
 *   censored [N] uint8 (non-zero = dropped), u [N] uniform numbers in [0, 1)
 *   (read for dropped workers only; the caller draws them), x_full [N] out,
 *   n_exceed [N] int32 out or NULL (m for dropped workers, -1 for observed):
 *   all dev.  workspace: dev, at least dkf_impute_workspace(S, N) bytes,
 *   4-byte aligned, contents are scratch.
 * Errors: DKF_EINVAL (NULL, S or N < 1, tau NaN, workspace too small),
 * DKF_EUNSUPPORTED (more than 2^40 entries), DKF_EHIP. */
int dkf_impute_censored(const float *samples, int32_t S, int32_t N, const float *x_obs, const uint8_t *censored,
                        float tau, const float *u, float *x_full, int32_t *n_exceed, void *workspace,
                        size_t workspace_bytes, void *stream);
size_t dkf_impute_workspace(int32_t S, int32_t N);

/* Filter state (window, normaliser, counters) as an opaque blob, so that a
 * run can be resumed.  get: *bytes in = capacity, out = size needed/written
 * (buf may be NULL to query).  Both synchronise the device. */
int dkf_get_state(const dkf_model *m, void *buf, size_t *bytes);
int dkf_set_state(dkf_model *m, const void *buf, size_t bytes);

/* Which kernels dkf_sample_runtimes / dkf_decide use for the sampling stage
 * (Sec. 3.1.3: guide chain, transition draw, emission draw).  All variants
 * compute the same thing to the same tolerance; the default picks by size.
 *   DKF_SAMPLER_AUTO    sixteen samples per workgroup up to 4096 samples where
 *                       that kernel is built for the layer sizes, four per
 *                       wavefront up to 8192, sixteen per wavefront above; the
 *                       staged kernels for bf16 models and for layer sizes the
 *                       fused kernels are not built for
 *   DKF_SAMPLER_WAVE16  one fused kernel, sixteen samples per wavefront
 *   DKF_SAMPLER_WAVE4   one fused kernel, four samples per wavefront
 *   DKF_SAMPLER_STAGED  guide/transition kernel + four GEMM kernels
 *   DKF_SAMPLER_SPLIT   one fused kernel, sixteen samples per workgroup, every
 *                       layer split over the workgroup's wavefronts
 * Returns DKF_EUNSUPPORTED (and changes nothing) if the model's sizes or dtype
 * rule the requested variant out.  Host call; takes effect at the next call. */
#define DKF_SAMPLER_AUTO 0
#define DKF_SAMPLER_WAVE16 1
#define DKF_SAMPLER_WAVE4 2
#define DKF_SAMPLER_STAGED 3
#define DKF_SAMPLER_SPLIT 4
int dkf_set_sampler(dkf_model *m, int32_t variant);

/* Which of the variants above a dkf_sample_runtimes / dkf_decide call with S samples
 * launches under the current setting (never DKF_SAMPLER_AUTO; DKF_SAMPLER_STAGED
 * stands for every path made of several kernels, bf16 models included).  Host
 * call, no device work.  DKF_EINVAL for a NULL model or S < 1. */
int dkf_sampler_in_use(const dkf_model *m, int32_t S);

/* Whether a dkf_decide call with S samples has the sampler sort the rows it draws
 * (order statistics of Sec. 3.1.1, last paragraph, taken before the samples leave
 * the compute unit: the decision then has no row-sort launch and reads no sample
 * back): 1 for DKF_SAMPLER_SPLIT with eight wavefronts per workgroup, 128 or 512
 * workers and S a multiple of 16, else 0.  dkf_sample_runtimes and cutoff_select
 * called separately always sort in cutoff_select.  Host call, no device work.
 * DKF_EINVAL for a NULL model or S < 1. */
int dkf_decide_sorts_in_sampler(const dkf_model *m, int32_t S);

/* Per-kernel timing with HIP events recorded on the stream the kernels are
 * launched on (process-wide, for benchmarks; not recorded inside dkf_decide's
 * captured graph).  Stage ids: 0 filter (projection + RNN chains), 1 guide
 * chain + transition, 2 emission mean hidden layer, 3 emission mean, 4
 * emission scale hidden layer, 5 emission scale + draw, 6 row sort + rank
 * sums, 7 rank means + argmax, 8 the fused sampler (stages 1-5 in one kernel, used
 * for the layer sizes it is built for; then stages 1-5 record nothing).
 * dkf_timing_enable(mask) starts recording for the stages in the bit mask (0
 * stops).  dkf_timing_read synchronises the device and returns, for one
 * stage, the number of launches recorded and their summed duration in
 * milliseconds, then clears that stage's records.  At most 4096 launches per
 * stage are kept between reads. */
#define DKF_NUM_STAGES 9
int dkf_timing_enable(uint32_t stage_mask);
int dkf_timing_read(int32_t stage, int32_t *launches, double *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* CUTOFF_DKF_H */
