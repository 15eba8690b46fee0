/*
 * CPU oracle for the Cutoff-SGD predictor: TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision restatement of what the paper's
 * predict_cutoff computes (Teng & Wood, "High Throughput Synchronous
 * Distributed SGD", Alg. 1 server loop; Sec. 3, 3.1.1-3.1.3).  Nothing in the
 * product path may call into this file; it shares no code with the GPU
 * library and exists so that tests, the smoke check and the benchmark's CPU
 * baseline have something independent to compare against.
 *
 * Every layer is written as  y = act(W x + b)  with W stored [out][in], one
 * loop nest per layer, no blocking, no fusion, no BLAS.  The only parallelism
 * is an OpenMP loop over the independent Monte-Carlo samples.
 *
 * Readings taken where the paper is silent or ambiguous are marked READING.
 *
 * Parity pins (tests, CPU only): closed-form order statistics of iid
 * uniform / exponential / normal rows, brute-force argmax on tiny N, the
 * paper's 10 s / 8 s example, degenerate-weight cases that collapse the
 * network to closed forms, hand-worked small cases with literal expected
 * values for the gate and the combiner at ordinary values, the all-widths-one
 * chain worked as scalar arithmetic by a math-only script, and an independent
 * numpy float64 transcription of the equations (an index check, not a pin).  The trained-model behaviour of the whole pipeline (the
 * paper's Fig. 2/3) is "parity unpinned": no trained weights, traces or
 * printed predictions exist to compare with.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_WARMUP 1
#define ORACLE_NO_ELIGIBLE 2
#define ORACLE_EINVAL (-1)
#define ORACLE_ENOTREADY (-2)
#define ORACLE_EBADOBS (-3)

typedef struct {
    int32_t n_workers, lag, z_dim, hidden, rnn_dim;
    int32_t emit_mean_act; /* 0: identity hidden layer in I (paper), 1: ReLU */
} oracle_config;

typedef struct {
    oracle_config cfg;
    /* inference network (Sec. 3.1.3, guide program) */
    double *rnn_f_w_ih, *rnn_f_b_ih, *rnn_f_w_hh, *rnn_f_b_hh;
    double *rnn_b_w_ih, *rnn_b_b_ih, *rnn_b_w_hh, *rnn_b_b_hh;
    double *comb_w, *comb_b, *mu_w, *mu_b, *sig_w, *sig_b, *z0;
    /* gated transition G, H */
    double *gate1_w, *gate1_b, *gate2_w, *gate2_b;
    double *prop1_w, *prop1_b, *prop2_w, *prop2_b;
    double *lin_w, *lin_b, *tscale_w, *tscale_b;
    /* emission I, J */
    double *emean1_w, *emean1_b, *emean2_w, *emean2_b;
    double *escale1_w, *escale1_b, *escale2_w, *escale2_b;
    double *store;
    /* mixed-precision mode (MLP matrices and MLP inputs rounded to bf16, everything else as before):
     * the same tensors as `store`, every value rounded; see oracle_set_mlp_bf16 */
    double *store_bf16;
    double *fold_w, *fold_b; /* [H][H], [H]: J's first layer applied to I's hidden vector, see oracle_set_mlp_bf16 */
    int mlp_bf16;
    /* fixed-lag window of raw observations, oldest first */
    double *window; /* [L][N] */
    int32_t count;  /* observations pushed so far (saturates at INT32_MAX) */
    double scale;   /* normaliser s; 0 until the first window is complete */
} oracle_model;

static size_t blob_floats(const oracle_config *c) {
    size_t N = c->n_workers, Z = c->z_dim, H = c->hidden, R = c->rnn_dim;
    size_t rnn = 2 * (R * N + R + R * R + R);
    size_t guide = R * Z + R + Z * R + Z + Z * Z + Z + Z;
    size_t trans = 2 * (H * Z + H + Z * H + Z) + 2 * (Z * Z + Z);
    size_t emit = H * Z + H + N * H + N + H * N + H + N * H + N;
    return rnn + guide + trans + emit;
}

size_t oracle_blob_bytes(const oracle_config *c) { return 32 + 4 * blob_floats(c); }

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

void oracle_free(oracle_model *m) {
    if (!m) return;
    free(m->store);
    free(m->store_bf16);
    free(m->fold_w);
    free(m->fold_b);
    free(m->window);
    free(m);
}

/* Weight blob: int32[8] header {magic 'DKFW', version, N, L, Z, H, R, 0}, then
 * fp32 tensors in the fixed order below, each matrix [out][in] row-major. */
oracle_model *oracle_load_weights(const oracle_config *c, const void *blob, size_t bytes) {
    if (!c || !blob) return NULL;
    if (c->n_workers < 1 || c->lag < 1 || c->z_dim < 1 || c->hidden < 1 || c->rnn_dim < 1) return NULL;
    if (bytes != oracle_blob_bytes(c)) return NULL;
    int32_t head[8];
    memcpy(head, blob, 32);
    if (head[0] != 0x57464B44 || head[1] != 1 || head[2] != c->n_workers || head[3] != c->lag ||
        head[4] != c->z_dim || head[5] != c->hidden || head[6] != c->rnn_dim)
        return NULL;
    oracle_model *m = (oracle_model *)calloc(1, sizeof *m);
    if (!m) return NULL;
    m->cfg = *c;
    size_t nf = blob_floats(c);
    m->store = (double *)malloc(nf * sizeof(double));
    m->window = (double *)calloc((size_t)c->lag * c->n_workers, sizeof(double));
    if (!m->store || !m->window) { oracle_free(m); return NULL; }
    const float *src = (const float *)((const char *)blob + 32);
    for (size_t i = 0; i < nf; ++i) m->store[i] = (double)src[i];
    size_t N = c->n_workers, Z = c->z_dim, H = c->hidden, R = c->rnn_dim;
    double *p = m->store;
#define TAKE(field, count) do { m->field = p; p += (count); } while (0)
    TAKE(rnn_f_w_ih, R * N); TAKE(rnn_f_b_ih, R); TAKE(rnn_f_w_hh, R * R); TAKE(rnn_f_b_hh, R);
    TAKE(rnn_b_w_ih, R * N); TAKE(rnn_b_b_ih, R); TAKE(rnn_b_w_hh, R * R); TAKE(rnn_b_b_hh, R);
    TAKE(comb_w, R * Z); TAKE(comb_b, R);
    TAKE(mu_w, Z * R); TAKE(mu_b, Z);
    TAKE(sig_w, Z * Z); TAKE(sig_b, Z);
    TAKE(z0, Z);
    TAKE(gate1_w, H * Z); TAKE(gate1_b, H); TAKE(gate2_w, Z * H); TAKE(gate2_b, Z);
    TAKE(prop1_w, H * Z); TAKE(prop1_b, H); TAKE(prop2_w, Z * H); TAKE(prop2_b, Z);
    TAKE(lin_w, Z * Z); TAKE(lin_b, Z);
    TAKE(tscale_w, Z * Z); TAKE(tscale_b, Z);
    TAKE(emean1_w, H * Z); TAKE(emean1_b, H); TAKE(emean2_w, N * H); TAKE(emean2_b, N);
    TAKE(escale1_w, H * N); TAKE(escale1_b, H); TAKE(escale2_w, N * H); TAKE(escale2_b, N);
#undef TAKE
    m->count = 0;
    m->scale = 0.0;
    return m;
}

void oracle_reset(oracle_model *m) {
    m->count = 0;
    m->scale = 0.0;
    memset(m->window, 0, sizeof(double) * (size_t)m->cfg.lag * m->cfg.n_workers);
}

double oracle_scale(const oracle_model *m) { return m->scale; }

/* ---- mixed precision: "MLPs in bf16 with fp32 accumulation" -------------------------------
 * bfloat16 keeps 8 significant bits (1 implicit + 7 stored) and the exponent range of fp32.
 * Round to nearest, ties to even, written from that definition (the default floating-point
 * rounding mode is to-nearest-even, which is what nearbyint applies).  Zero, infinities and NaN
 * pass through; the exponent range is not clamped (no value here comes near its ends). */
double oracle_round_bf16(double v) {
    if (v == 0.0 || !isfinite(v)) return v;
    int e;
    double f = frexp(v, &e);                       /* v = f 2^e, 0.5 <= |f| < 1 */
    return ldexp(nearbyint(ldexp(f, 8)), e - 8);   /* 8 significant bits */
}

/* Switch the mixed-precision mode of the sampler on or off (off after loading).
 * READING of "MLPs in bf16 with fp32 accumulation": every MLP matrix (guide: combiner, mean,
 * scale; transition; emission) and every vector that is multiplied by one is rounded to bf16;
 * sums, biases, nonlinearities, the noise mix and all outputs are not rounded (here: double, the
 * kernel: fp32); the RNN encoders are not MLPs and stay in full precision.  In the guide's mean,
 * K(h_out) with h_out = (tanh(.) + h_left + h_right)/3 is linear, so the encodings' share
 * W (h_left + h_right)/3 + b is the same for every sample: it is formed once per window position
 * in full precision with the unrounded matrix, and only the per-sample term W tanh(.)/3 is a
 * product of rounded operands.  Likewise in the emission: I ends in a linear layer, mean = W2 h + b2,
 * and J's first layer is linear in the mean, so J's hidden pre-activation is
 * W1' mean + b1' = (W1' W2) h + (W1' b2 + b1'): the H x H matrix W1' W2 is formed once from the
 * unrounded matrices, then rounded like any other matrix, and multiplies the rounded h; the bias
 * W1' b2 + b1' is not rounded.  The mean itself, W2 h + b2, stays a product of rounded operands.
 * (With rounding off none of this applies: every layer is evaluated as the paper writes it.) */
int oracle_set_mlp_bf16(oracle_model *m, int on) {
    if (on && !m->store_bf16) {
        size_t nf = blob_floats(&m->cfg);
        size_t N = m->cfg.n_workers, H = m->cfg.hidden;
        m->store_bf16 = (double *)malloc(nf * sizeof(double));
        m->fold_w = (double *)malloc(H * H * sizeof(double));
        m->fold_b = (double *)malloc(H * sizeof(double));
        if (!m->store_bf16 || !m->fold_w || !m->fold_b) return ORACLE_EINVAL;
        for (size_t i = 0; i < nf; ++i) m->store_bf16[i] = oracle_round_bf16(m->store[i]);
        for (size_t o = 0; o < H; ++o) {
            for (size_t i = 0; i < H; ++i) {
                double acc = 0.0;
                for (size_t n = 0; n < N; ++n) acc += m->escale1_w[o * N + n] * m->emean2_w[n * H + i];
                m->fold_w[o * H + i] = oracle_round_bf16(acc);
            }
            double acc = m->escale1_b[o];
            for (size_t n = 0; n < N; ++n) acc += m->escale1_w[o * N + n] * m->emean2_b[n];
            m->fold_b[o] = acc;
        }
    }
    m->mlp_bf16 = on ? 1 : 0;
    return ORACLE_OK;
}

/* ---- elementary functions ------------------------------------------------ */

static double relu(double v) { return v > 0.0 ? v : 0.0; }
static double softplus(double v) { return (v > 0.0 ? v : 0.0) + log1p(exp(-fabs(v))); }
static double sigmoid(double v) {
    if (v >= 0.0) return 1.0 / (1.0 + exp(-v));
    double e = exp(v);
    return e / (1.0 + e);
}

/* y[out] = W[out][in] x + b */
static void affine(const double *W, const double *b, const double *x, int n_in, int n_out, double *y) {
    for (int o = 0; o < n_out; ++o) {
        double acc = b[o];
        for (int i = 0; i < n_in; ++i) acc += W[(size_t)o * n_in + i] * x[i];
        y[o] = acc;
    }
}

/* One MLP layer y = W x + b in the model's precision mode: full precision, or (mixed precision) the
 * matrix and the input vector rounded to bf16, the sum and the bias not.  W must point into
 * m->store; xq is scratch for the rounded input (at least n_in doubles). */
static void mlp_layer(const oracle_model *m, const double *W, const double *b, const double *x, int n_in,
                      int n_out, double *y, double *xq) {
    if (!m->mlp_bf16) {
        affine(W, b, x, n_in, n_out, y);
        return;
    }
    const double *Wq = m->store_bf16 + (W - m->store);
    for (int i = 0; i < n_in; ++i) xq[i] = oracle_round_bf16(x[i]);
    affine(Wq, b, xq, n_in, n_out, y);
}

/* ---- fixed-lag window and normaliser (Sec. 3.1.2; end of Sec. 3.1.3) ------ */

/* Append one observed N-vector of run-times (seconds).  The window holds the
 * last L vectors.  READING: the normaliser is one scalar, twice the mean of
 * the first complete window, fixed from then on.  Returns ORACLE_WARMUP until
 * L vectors have been seen. */
int oracle_filter_step(oracle_model *m, const double *x_obs) {
    int N = m->cfg.n_workers, L = m->cfg.lag;
    for (int j = 0; j < N; ++j)
        if (!isfinite(x_obs[j]) || !(x_obs[j] > 0.0)) return ORACLE_EBADOBS;
    if (m->count >= L) memmove(m->window, m->window + N, sizeof(double) * (size_t)(L - 1) * N);
    int slot = m->count < L ? m->count : L - 1;
    memcpy(m->window + (size_t)slot * N, x_obs, sizeof(double) * N);
    if (m->count < INT32_MAX) m->count++;
    if (m->count == L) {
        double sum = 0.0;
        for (size_t i = 0; i < (size_t)L * N; ++i) sum += m->window[i];
        m->scale = 2.0 * sum / ((double)L * N);
    }
    return m->count < L ? ORACLE_WARMUP : ORACLE_OK;
}

/* The RNN encodings of the guide (Sec. 3.1.3): h_left runs forward over the
 * window from a zero state, h_right backward.  READING: single-layer Elman
 * cells with ReLU, h_t = ReLU(W_ih x_t + b_ih + W_hh h_prev + b_hh); the
 * encodings at position t include x_t on both sides.  hl, hr: [L][R]. */
int oracle_encode_window(const oracle_model *m, double *hl, double *hr) {
    int N = m->cfg.n_workers, L = m->cfg.lag, R = m->cfg.rnn_dim;
    if (m->count < L) return ORACLE_ENOTREADY;
    double *xn = (double *)malloc(sizeof(double) * N);
    double *a = (double *)malloc(sizeof(double) * R);
    double *b = (double *)malloc(sizeof(double) * R);
    double *prev = (double *)malloc(sizeof(double) * R);
    for (int dir = 0; dir < 2; ++dir) {
        const double *w_ih = dir ? m->rnn_b_w_ih : m->rnn_f_w_ih, *b_ih = dir ? m->rnn_b_b_ih : m->rnn_f_b_ih;
        const double *w_hh = dir ? m->rnn_b_w_hh : m->rnn_f_w_hh, *b_hh = dir ? m->rnn_b_b_hh : m->rnn_f_b_hh;
        double *out = dir ? hr : hl;
        for (int r = 0; r < R; ++r) prev[r] = 0.0;
        for (int step = 0; step < L; ++step) {
            int t = dir ? L - 1 - step : step;
            for (int j = 0; j < N; ++j) xn[j] = m->window[(size_t)t * N + j] / m->scale;
            affine(w_ih, b_ih, xn, N, R, a);
            affine(w_hh, b_hh, prev, R, R, b);
            for (int r = 0; r < R; ++r) prev[r] = relu(a[r] + b[r]);
            memcpy(out + (size_t)t * R, prev, sizeof(double) * R);
        }
    }
    free(xn); free(a); free(b); free(prev);
    return ORACLE_OK;
}

/* ---- one Monte-Carlo sample (Sec. 3.1.3, posterior-predictive approximation) */

typedef struct { double *r1, *r2, *z, *mu, *pre, *zn, *g, *h, *lin, *G, *hid, *mean, *sd, *xq; } scratch;

static scratch scratch_new(const oracle_config *c) {
    scratch s;
    int N = c->n_workers, Z = c->z_dim, H = c->hidden, R = c->rnn_dim;
    int big = H > R ? H : R;
    s.r1 = (double *)malloc(sizeof(double) * big);
    s.r2 = (double *)malloc(sizeof(double) * big);
    s.hid = (double *)malloc(sizeof(double) * big);
    s.z = (double *)malloc(sizeof(double) * Z);
    s.mu = (double *)malloc(sizeof(double) * Z);
    s.pre = (double *)malloc(sizeof(double) * Z);
    s.zn = (double *)malloc(sizeof(double) * Z);
    s.g = (double *)malloc(sizeof(double) * Z);
    s.h = (double *)malloc(sizeof(double) * Z);
    s.lin = (double *)malloc(sizeof(double) * Z);
    s.G = (double *)malloc(sizeof(double) * Z);
    s.mean = (double *)malloc(sizeof(double) * N);
    s.sd = (double *)malloc(sizeof(double) * N);
    int widest = big > N ? big : N;
    if (Z > widest) widest = Z;
    s.xq = (double *)malloc(sizeof(double) * widest);
    return s;
}

static void scratch_free(scratch *s) {
    free(s->r1); free(s->r2); free(s->hid); free(s->z); free(s->mu); free(s->pre); free(s->zn);
    free(s->g); free(s->h); free(s->lin); free(s->G); free(s->mean); free(s->sd); free(s->xq);
}

/* Optional taps on the inside of the gated transition of one sample (any may be NULL). */
typedef struct {
    double *gate_hidden; /* [H] W_g1 z_T + b, before the ReLU */
    double *gate_pre;    /* [Z] argument of the sigmoid */
    double *gate;        /* [Z] g */
    double *lin;         /* [Z] W_l z_T + b_l */
    double *prop;        /* [Z] proposed mean h */
    double *G;           /* [Z] transition mean */
    double *Hs;          /* [Z] transition scale */
} transition_taps;

/* Encodings that enter h_out at window position t.  READING: h_left covers the observations up to
 * and including x_t, h_right those from x_t on.  As printed (h_left over x_{T-l:t-1}, h_right over
 * x_{t+1:T}) neither would contain x_t, so the last latent z_T would never see the newest
 * observation; building with -DORACLE_A8_LITERAL gives that literal reading (an index shift, zero
 * state at the window's ends) for the test that shows the difference. */
#ifdef ORACLE_A8_LITERAL
#define H_LEFT(t, r) ((t) > 0 ? hl[((size_t)(t) - 1) * R + (r)] : 0.0)
#define H_RIGHT(t, r) ((t) < L - 1 ? hr[((size_t)(t) + 1) * R + (r)] : 0.0)
#else
#define H_LEFT(t, r) hl[(size_t)(t) * R + (r)]
#define H_RIGHT(t, r) hr[(size_t)(t) * R + (r)]
#endif

static void sample_one(const oracle_model *m, const double *hl, const double *hr, int S, int k,
                       const float *eps_q, const float *eps_z, const float *eps_x, scratch *w,
                       double *x_out, double *zT_out, double *zn_out, double *mean_out, double *sd_out,
                       const transition_taps *tap) {
    int N = m->cfg.n_workers, L = m->cfg.lag, Z = m->cfg.z_dim, H = m->cfg.hidden, R = m->cfg.rnn_dim;
    /* Guide chain: z_t ~ N(mu_q, sigma_q) for t = 1..L, sequential in t.
     * READING: the latent before the window is a learned vector z0. */
    for (int i = 0; i < Z; ++i) w->z[i] = m->z0[i];
    for (int t = 0; t < L; ++t) {
        mlp_layer(m, m->comb_w, m->comb_b, w->z, Z, R, w->r1, w->xq);
        if (!m->mlp_bf16) {
            for (int r = 0; r < R; ++r)
                w->r2[r] = (tanh(w->r1[r]) + H_LEFT(t, r) + H_RIGHT(t, r)) / 3.0; /* h_out */
            affine(m->mu_w, m->mu_b, w->r2, R, Z, w->mu);                                     /* mu_q = K(h_out) */
        } else {
            /* the same K(h_out), split as oracle_set_mlp_bf16 describes */
            const double *Wq = m->store_bf16 + (m->mu_w - m->store);
            for (int r = 0; r < R; ++r) w->xq[r] = oracle_round_bf16(tanh(w->r1[r]));
            for (int i = 0; i < Z; ++i) {
                double per_sample = 0.0, context = 0.0;
                for (int r = 0; r < R; ++r) {
                    per_sample += Wq[(size_t)i * R + r] * w->xq[r];
                    context += m->mu_w[(size_t)i * R + r] * (H_LEFT(t, r) + H_RIGHT(t, r));
                }
                w->mu[i] = per_sample / 3.0 + (context / 3.0 + m->mu_b[i]);
            }
        }
        mlp_layer(m, m->sig_w, m->sig_b, w->mu, Z, Z, w->pre, w->xq);                         /* sigma_q = L(mu_q) */
        for (int i = 0; i < Z; ++i) {
            double sigma = softplus(w->pre[i]);
            /* READING: the second argument of N(.,.) is a standard deviation */
            w->z[i] = w->mu[i] + sigma * (double)eps_q[((size_t)t * S + k) * Z + i];
        }
    }
    if (zT_out) memcpy(zT_out, w->z, sizeof(double) * Z);
    /* Gated transition z_{T+1} ~ N(G(z_T), H(z_T)) */
    mlp_layer(m, m->gate1_w, m->gate1_b, w->z, Z, H, w->hid, w->xq);
    if (tap && tap->gate_hidden) memcpy(tap->gate_hidden, w->hid, sizeof(double) * H);
    for (int i = 0; i < H; ++i) w->hid[i] = relu(w->hid[i]);
    mlp_layer(m, m->gate2_w, m->gate2_b, w->hid, H, Z, w->g, w->xq);
    if (tap && tap->gate_pre) memcpy(tap->gate_pre, w->g, sizeof(double) * Z);
    for (int i = 0; i < Z; ++i) w->g[i] = sigmoid(w->g[i]);
    mlp_layer(m, m->prop1_w, m->prop1_b, w->z, Z, H, w->hid, w->xq);
    for (int i = 0; i < H; ++i) w->hid[i] = relu(w->hid[i]);
    mlp_layer(m, m->prop2_w, m->prop2_b, w->hid, H, Z, w->h, w->xq);
    mlp_layer(m, m->lin_w, m->lin_b, w->z, Z, Z, w->lin, w->xq);
    for (int i = 0; i < Z; ++i) w->G[i] = (1.0 - w->g[i]) * w->lin[i] + w->g[i] * w->h[i];
    for (int i = 0; i < Z; ++i) w->mu[i] = relu(w->G[i]);
    mlp_layer(m, m->tscale_w, m->tscale_b, w->mu, Z, Z, w->pre, w->xq);
    for (int i = 0; i < Z; ++i) w->pre[i] = softplus(w->pre[i]);
    for (int i = 0; i < Z; ++i) w->zn[i] = w->G[i] + w->pre[i] * (double)eps_z[(size_t)k * Z + i];
    if (zn_out) memcpy(zn_out, w->zn, sizeof(double) * Z);
    if (tap) {
        if (tap->gate) memcpy(tap->gate, w->g, sizeof(double) * Z);
        if (tap->lin) memcpy(tap->lin, w->lin, sizeof(double) * Z);
        if (tap->prop) memcpy(tap->prop, w->h, sizeof(double) * Z);
        if (tap->G) memcpy(tap->G, w->G, sizeof(double) * Z);
        if (tap->Hs) memcpy(tap->Hs, w->pre, sizeof(double) * Z);
    }
    /* Emission x_{T+1} ~ N(I(z_{T+1}), J(z_{T+1})), J fed by I's output */
    mlp_layer(m, m->emean1_w, m->emean1_b, w->zn, Z, H, w->hid, w->xq);
    if (m->cfg.emit_mean_act == 1)
        for (int i = 0; i < H; ++i) w->hid[i] = relu(w->hid[i]);
    mlp_layer(m, m->emean2_w, m->emean2_b, w->hid, H, N, w->mean, w->xq);
    if (!m->mlp_bf16) {
        mlp_layer(m, m->escale1_w, m->escale1_b, w->mean, N, H, w->hid, w->xq);
    } else {
        /* the same layer on I's hidden vector, as oracle_set_mlp_bf16 describes */
        for (int i = 0; i < H; ++i) w->xq[i] = oracle_round_bf16(w->hid[i]);
        affine(m->fold_w, m->fold_b, w->xq, H, H, w->hid);
    }
    for (int i = 0; i < H; ++i) w->hid[i] = relu(w->hid[i]);
    mlp_layer(m, m->escale2_w, m->escale2_b, w->hid, H, N, w->sd, w->xq);
    for (int j = 0; j < N; ++j) {
        w->sd[j] = softplus(w->sd[j]);
        /* back to seconds: the model lives in units of the normaliser */
        x_out[j] = m->scale * (w->mean[j] + w->sd[j] * (double)eps_x[(size_t)k * N + j]);
    }
    if (mean_out) memcpy(mean_out, w->mean, sizeof(double) * N);
    if (sd_out) memcpy(sd_out, w->sd, sizeof(double) * N);
}

/* Draw run-time vectors for the samples listed in `rows` (or all S samples
 * when rows == NULL, then n_rows is ignored).  Noise tensors are inputs:
 * eps_q [L][S][Z], eps_z [S][Z], eps_x [S][N], fp32 standard normals.
 * Outputs are [n_out][.] in the order of `rows`; optional ones may be NULL. */
int oracle_sample_runtimes(const oracle_model *m, int S, const int32_t *rows, int n_rows,
                           const float *eps_q, const float *eps_z, const float *eps_x,
                           double *out_samples, double *out_zT, double *out_znext,
                           double *out_mean, double *out_sd) {
    int N = m->cfg.n_workers, L = m->cfg.lag, Z = m->cfg.z_dim, R = m->cfg.rnn_dim;
    if (S < 1 || !eps_q || !eps_z || !eps_x || !out_samples) return ORACLE_EINVAL;
    if (m->count < L) return ORACLE_ENOTREADY;
    int n_out = rows ? n_rows : S;
    for (int i = 0; rows && i < n_rows; ++i)
        if (rows[i] < 0 || rows[i] >= S) return ORACLE_EINVAL;
    double *hl = (double *)malloc(sizeof(double) * (size_t)L * R);
    double *hr = (double *)malloc(sizeof(double) * (size_t)L * R);
    oracle_encode_window(m, hl, hr);
#pragma omp parallel
    {
        scratch w = scratch_new(&m->cfg);
#pragma omp for schedule(static)
        for (int i = 0; i < n_out; ++i) {
            int k = rows ? rows[i] : i;
            sample_one(m, hl, hr, S, k, eps_q, eps_z, eps_x, &w, out_samples + (size_t)i * N,
                       out_zT ? out_zT + (size_t)i * Z : NULL, out_znext ? out_znext + (size_t)i * Z : NULL,
                       out_mean ? out_mean + (size_t)i * N : NULL, out_sd ? out_sd + (size_t)i * N : NULL, NULL);
        }
        scratch_free(&w);
    }
    free(hl); free(hr);
    return ORACLE_OK;
}

/* The inside of the gated transition (Sec. 3.1.3: g, h, G, H of the transition display) for the
 * samples listed in `rows` (all S when rows == NULL): the same sample_one as above with its taps
 * switched on.  Outputs [n_out][H] (gate_hidden) or [n_out][Z]; any may be NULL. */
int oracle_transition_terms(const oracle_model *m, int S, const int32_t *rows, int n_rows,
                            const float *eps_q, const float *eps_z, const float *eps_x,
                            double *out_gate_hidden, double *out_gate_pre, double *out_gate,
                            double *out_lin, double *out_prop, double *out_G, double *out_Hs) {
    int N = m->cfg.n_workers, L = m->cfg.lag, Z = m->cfg.z_dim, H = m->cfg.hidden, R = m->cfg.rnn_dim;
    if (S < 1 || !eps_q || !eps_z || !eps_x) return ORACLE_EINVAL;
    if (m->count < L) return ORACLE_ENOTREADY;
    int n_out = rows ? n_rows : S;
    for (int i = 0; rows && i < n_rows; ++i)
        if (rows[i] < 0 || rows[i] >= S) return ORACLE_EINVAL;
    double *hl = (double *)malloc(sizeof(double) * (size_t)L * R);
    double *hr = (double *)malloc(sizeof(double) * (size_t)L * R);
    oracle_encode_window(m, hl, hr);
#pragma omp parallel
    {
        scratch w = scratch_new(&m->cfg);
        double *x = (double *)malloc(sizeof(double) * N);
#pragma omp for schedule(static)
        for (int i = 0; i < n_out; ++i) {
            int k = rows ? rows[i] : i;
            transition_taps tap;
            tap.gate_hidden = out_gate_hidden ? out_gate_hidden + (size_t)i * H : NULL;
            tap.gate_pre = out_gate_pre ? out_gate_pre + (size_t)i * Z : NULL;
            tap.gate = out_gate ? out_gate + (size_t)i * Z : NULL;
            tap.lin = out_lin ? out_lin + (size_t)i * Z : NULL;
            tap.prop = out_prop ? out_prop + (size_t)i * Z : NULL;
            tap.G = out_G ? out_G + (size_t)i * Z : NULL;
            tap.Hs = out_Hs ? out_Hs + (size_t)i * Z : NULL;
            sample_one(m, hl, hr, S, k, eps_q, eps_z, eps_x, &w, x, NULL, NULL, NULL, NULL, &tap);
        }
        free(x);
        scratch_free(&w);
    }
    free(hl); free(hr);
    return ORACLE_OK;
}

/* ---- noise the sampler may draw itself ------------------------------------------
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) written from its published definition:
 * ten rounds of  (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0))
 * with M0 = 0xD2511F53, M1 = 0xCD9E8D57, the key raised by (0x9E3779B9, 0xBB67AE85) after
 * every round.  READING (the paper does not say how its samples are drawn): element i of
 * tensor t uses counter (i/4 low, i/4 high, t, 0) and key (seed low, seed high); the four
 * output words give two Box-Muller pairs from 24-bit uniforms u1 = ((w>>8)+1)/2^24,
 * u2 = (w>>8)/2^24. */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

void oracle_fill_normal(uint64_t seed, uint32_t tensor, size_t n, float *out) {
    const double two_pi = 6.283185307179586476925286766559;
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (size_t g = 0; g * 4 < n; ++g) {
        uint32_t ctr[4] = {(uint32_t)g, (uint32_t)((uint64_t)g >> 32), tensor, 0u}, w[4];
        oracle_philox4x32_10(ctr, key, w);
        double v[4];
        for (int pair = 0; pair < 2; ++pair) {
            double u1 = (double)((w[2 * pair] >> 8) + 1u) / 16777216.0;
            double u2 = (double)(w[2 * pair + 1] >> 8) / 16777216.0;
            double r = sqrt(-2.0 * log(u1));
            v[2 * pair] = r * cos(two_pi * u2);
            v[2 * pair + 1] = r * sin(two_pi * u2);
        }
        for (int j = 0; j < 4 && g * 4 + j < n; ++j) out[g * 4 + j] = (float)v[j];
    }
}

/* ---- Monte-Carlo order statistics and the cutoff (Sec. 3; Sec. 3.1.1) ------ */

typedef struct { double v; int32_t idx; } keyed;

/* READING: ties are ordered -0 before +0, NaN last, then by worker index, so
 * the permutation is unique. */
static int keyed_cmp(const void *pa, const void *pb) {
    const keyed *a = (const keyed *)pa, *b = (const keyed *)pb;
    int na = isnan(a->v), nb = isnan(b->v);
    if (na != nb) return na ? 1 : -1;
    if (!na) {
        if (a->v < b->v) return -1;
        if (a->v > b->v) return 1;
        int sa = signbit(a->v) != 0, sb = signbit(b->v) != 0;
        if (sa != sb) return sa ? -1 : 1;
    }
    return (a->idx > b->idx) - (a->idx < b->idx);
}

/* samples [S][N]: sort every row ascending (Monte-Carlo order statistics, Sec. 3.1.1 last paragraph), average
 * each rank over the S rows, form Omega(c) = c / mean x_(c) and return the
 * maximiser, 1-based.  READING: only c in [c_min, c_max] whose mean exceeds
 * t_floor are eligible; ties go to the largest c; with nothing eligible the
 * answer is c_max and the status ORACLE_NO_ELIGIBLE.
 * out_sorted [S][N], out_perm [S][N] (0-based worker per rank), out_mean [N],
 * out_omega [N] (-inf where ineligible) are optional. */
int oracle_cutoff_select(const double *samples, int S, int N, int c_min, int c_max, double t_floor,
                         double *out_sorted, int32_t *out_perm, double *out_mean, double *out_omega,
                         int32_t *out_cstar) {
    if (!samples || !out_cstar || S < 1 || N < 1 || c_min < 1 || c_max > N || c_min > c_max) return ORACLE_EINVAL;
    double *sum = (double *)calloc(N, sizeof(double));
    keyed *row = (keyed *)malloc(sizeof(keyed) * N);
    for (int k = 0; k < S; ++k) {
        for (int j = 0; j < N; ++j) { row[j].v = samples[(size_t)k * N + j]; row[j].idx = j; }
        qsort(row, N, sizeof(keyed), keyed_cmp);
        for (int c = 0; c < N; ++c) {
            sum[c] += row[c].v;
            if (out_sorted) out_sorted[(size_t)k * N + c] = row[c].v;
            if (out_perm) out_perm[(size_t)k * N + c] = row[c].idx;
        }
    }
    int best = -1;
    double best_omega = -INFINITY;
    for (int c = 1; c <= N; ++c) {
        double mean = sum[c - 1] / (double)S;
        double omega = -INFINITY;
        if (c >= c_min && c <= c_max && mean > t_floor) omega = (double)c / mean;
        if (out_mean) out_mean[c - 1] = mean;
        if (out_omega) out_omega[c - 1] = omega;
        if (omega > -INFINITY && omega >= best_omega) { best_omega = omega; best = c; }
    }
    free(sum); free(row);
    if (best < 0) { *out_cstar = c_max; return ORACLE_NO_ELIGIBLE; }
    *out_cstar = best;
    return ORACLE_OK;
}

/* The other reading of "expected gradients per second" (Sec. 3, definition of Omega): the
 * expectation of the ratio, Omega(c) = E[c / x_(c)], estimated by the mean over the sampled rows of
 * c / x^(k)_(c), instead of the ratio of c to the expected order statistic.  READING: a rank is
 * eligible only if every sampled value of it exceeds t_floor >= 0 (a reciprocal of a non-positive
 * time means nothing); bounds, ties and the no-eligible case as in oracle_cutoff_select.
 * out_rate [N]: mean_k 1 / x^(k)_(c), +inf where some sample is <= t_floor; out_omega [N]: c * rate,
 * -inf where ineligible.  Both optional. */
int oracle_cutoff_select_rate(const double *samples, int S, int N, int c_min, int c_max, double t_floor,
                              double *out_rate, double *out_omega, int32_t *out_cstar) {
    if (!samples || !out_cstar || S < 1 || N < 1 || c_min < 1 || c_max > N || c_min > c_max) return ORACLE_EINVAL;
    if (!(t_floor >= 0.0)) return ORACLE_EINVAL;
    double *sum = (double *)calloc(N, sizeof(double));
    keyed *row = (keyed *)malloc(sizeof(keyed) * N);
    for (int k = 0; k < S; ++k) {
        for (int j = 0; j < N; ++j) { row[j].v = samples[(size_t)k * N + j]; row[j].idx = j; }
        qsort(row, N, sizeof(keyed), keyed_cmp);
        for (int c = 0; c < N; ++c) sum[c] += row[c].v > t_floor ? 1.0 / row[c].v : INFINITY;
    }
    int best = -1;
    double best_omega = -INFINITY;
    for (int c = 1; c <= N; ++c) {
        double rate = sum[c - 1] / (double)S;
        double omega = -INFINITY;
        if (c >= c_min && c <= c_max && isfinite(rate)) omega = (double)c * rate;
        if (out_rate) out_rate[c - 1] = rate;
        if (out_omega) out_omega[c - 1] = omega;
        if (omega > -INFINITY && omega >= best_omega) { best_omega = omega; best = c; }
    }
    free(sum); free(row);
    if (best < 0) { *out_cstar = c_max; return ORACLE_NO_ELIGIBLE; }
    *out_cstar = best;
    return ORACLE_OK;
}

/* Same, for an fp32 sample matrix (what the GPU hands over): every float is
 * exactly representable as a double, so order and ties are unchanged. */
int oracle_cutoff_select_f32(const float *samples, int S, int N, int c_min, int c_max, double t_floor,
                             double *out_sorted, int32_t *out_perm, double *out_mean, double *out_omega,
                             int32_t *out_cstar) {
    if (!samples || S < 1 || N < 1) return ORACLE_EINVAL;
    double *wide = (double *)malloc(sizeof(double) * (size_t)S * N);
    for (size_t i = 0; i < (size_t)S * N; ++i) wide[i] = (double)samples[i];
    int rc = oracle_cutoff_select(wide, S, N, c_min, c_max, t_floor, out_sorted, out_perm, out_mean, out_omega, out_cstar);
    free(wide);
    return rc;
}

/* The whole decision for the current window: sample, sort, average, argmax. */
int oracle_predict_cutoff(const oracle_model *m, int S, const float *eps_q, const float *eps_z,
                          const float *eps_x, int c_min, int c_max, double t_floor, int32_t *out_cstar) {
    int N = m->cfg.n_workers;
    if (S < 1) return ORACLE_EINVAL;
    double *x = (double *)malloc(sizeof(double) * (size_t)S * N);
    int rc = oracle_sample_runtimes(m, S, NULL, 0, eps_q, eps_z, eps_x, x, NULL, NULL, NULL, NULL);
    if (rc == ORACLE_OK) rc = oracle_cutoff_select(x, S, N, c_min, c_max, t_floor, NULL, NULL, NULL, NULL, out_cstar);
    free(x);
    return rc;
}

/* ---------------------------------------------------------------------------
 * Censored run-times (Sec. 4.2, "Handling Censored Run-times").
 *
 * After a cutoff the server has killed the stragglers, so their run-times are
 * only known to exceed the censoring time tau = the c-th arrival.  The filter
 * needs a full vector, so every dropped worker gets a value drawn from its
 * predictive run-time distribution left-truncated at tau (the display of
 * Sec. 4.2).
 * READING: the predictive distribution of worker w is represented by the S
 * Monte-Carlo draws samples[.][w] made for this iteration; the truncated
 * distribution is therefore the empirical distribution of the draws that
 * exceed tau, and one of them is picked with the supplied uniform number:
 * the floor(u * m)-th in sample order, m = number of exceeding draws.
 * READING: if no draw exceeds tau the smallest value consistent with the
 * censoring, tau itself, is used.
 * Observed workers keep their observed value.  n_exceed (optional) receives
 * m for dropped workers and -1 for observed ones.
 */
int oracle_impute_censored(const float *samples, int S, int N, const float *x_obs, const uint8_t *censored,
                           float tau, const float *u, float *x_full, int32_t *n_exceed) {
    if (!samples || !x_obs || !censored || !u || !x_full || S < 1 || N < 1) return ORACLE_EINVAL;
    for (int w = 0; w < N; ++w) {
        if (!censored[w]) {
            x_full[w] = x_obs[w];
            if (n_exceed) n_exceed[w] = -1;
            continue;
        }
        if (!(u[w] >= 0.0f && u[w] < 1.0f)) return ORACLE_EINVAL;
        int m = 0;
        for (int k = 0; k < S; ++k)
            if (samples[(size_t)k * N + w] > tau) ++m;
        if (n_exceed) n_exceed[w] = m;
        if (m == 0) { x_full[w] = tau; continue; }
        long pick = (long)floor((double)u[w] * (double)m);
        if (pick > m - 1) pick = m - 1;
        long seen = 0;
        for (int k = 0; k < S; ++k) {
            float v = samples[(size_t)k * N + w];
            if (v > tau) {
                if (seen == pick) { x_full[w] = v; break; }
                ++seen;
            }
        }
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Comparison cutoffs (Sec. 3.1.1 and Sec. 4).
 *
 * Standard normal quantile by bisection on the distribution function
 * Phi(x) = erfc(-x / sqrt 2) / 2: slow and obviously right. */
static double normal_quantile(double p) {
    if (!(p > 0.0)) return -INFINITY;
    if (!(p < 1.0)) return INFINITY;
    double lo = -40.0, hi = 40.0;
    for (int it = 0; it < 200; ++it) {
        double mid = 0.5 * (lo + hi);
        double cdf = 0.5 * erfc(-mid / sqrt(2.0));
        if (cdf < p) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

/* Elfving's approximation of the expected j-th of n iid normal order
 * statistics (eq. 4):  mu + sigma * Phi^-1((j - pi/8) / (n - pi/4 + 1)).
 * READING: the fraction is printed upside down in eq. 4; this is the form of
 * the cited source, and the only one that reproduces the value the paper
 * computes with it in Sec. 4.1. */
double oracle_elfving_mean(int j, int n, double mu, double sigma) {
    const double pi = 3.14159265358979323846;
    return mu + sigma * normal_quantile(((double)j - pi / 8.0) / ((double)n - pi / 4.0 + 1.0));
}

/* The "order" baseline of Sec. 4: the cutoff that maximises c / E[x_(c)] when
 * the order statistics are those of n iid normal run-times (Elfving).  Same
 * range, floor and tie rules as oracle_cutoff_select. */
int oracle_cutoff_elfving(int n, double mu, double sigma, int c_min, int c_max, double t_floor,
                          double *out_mean, double *out_omega, int32_t *out_cstar) {
    if (!out_cstar || n < 1 || c_min < 1 || c_max > n || c_min > c_max || !(sigma >= 0.0)) return ORACLE_EINVAL;
    int best = -1;
    double best_omega = -INFINITY;
    for (int c = 1; c <= n; ++c) {
        double mean = oracle_elfving_mean(c, n, mu, sigma);
        double omega = -INFINITY;
        if (c >= c_min && c <= c_max && mean > t_floor) omega = (double)c / mean;
        if (out_mean) out_mean[c - 1] = mean;
        if (out_omega) out_omega[c - 1] = omega;
        if (omega > -INFINITY && omega >= best_omega) { best_omega = omega; best = c; }
    }
    if (best < 0) { *out_cstar = c_max; return ORACLE_NO_ELIGIBLE; }
    *out_cstar = best;
    return ORACLE_OK;
}

static int dbl_cmp(const void *a, const void *b) {
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

/* Gradient throughput of a run over a recorded trace (Sec. 3, Omega; Fig. 2):
 * with cutoff c_t at iteration t the server waits for the c_t-th fastest
 * worker, so the run computes sum_t c_t gradients in sum_t x_{t,(c_t)} seconds.
 *   out[0] = that ratio for the given cutoffs,
 *   out[1] = full synchronisation, c_t = N,
 *   out[2] = the best cutoff in hindsight at every iteration, c_t = argmax_c c / x_{t,(c)}
 *            (the "maximum" curve of Fig. 2). */
int oracle_trace_throughput(const double *trace, int T, int N, const int32_t *cutoffs, double *out) {
    if (!trace || !cutoffs || !out || T < 1 || N < 1) return ORACLE_EINVAL;
    double *row = (double *)malloc(sizeof(double) * N);
    double g_cut = 0, t_cut = 0, g_sync = 0, t_sync = 0, g_best = 0, t_best = 0;
    for (int t = 0; t < T; ++t) {
        if (cutoffs[t] < 1 || cutoffs[t] > N) { free(row); return ORACLE_EINVAL; }
        memcpy(row, trace + (size_t)t * N, sizeof(double) * N);
        qsort(row, N, sizeof(double), dbl_cmp);
        g_cut += cutoffs[t];  t_cut += row[cutoffs[t] - 1];
        g_sync += N;          t_sync += row[N - 1];
        int best = 1;
        for (int c = 2; c <= N; ++c)
            if ((double)c / row[c - 1] >= (double)best / row[best - 1]) best = c;
        g_best += best;       t_best += row[best - 1];
    }
    free(row);
    out[0] = g_cut / t_cut; out[1] = g_sync / t_sync; out[2] = g_best / t_best;
    return ORACLE_OK;
}

/* Spread of the predicted order statistics (Fig. 3 draws every predicted
 * order statistic with a band of two standard deviations): sort every row of
 * samples [S][N] ascending; for each rank c the mean over the S rows and
 *   sd(c) = sqrt( (1/S) sum_k (x_(c),k - mean(c))^2 ).
 * READING: the paper does not say which normalisation its bands use; the plain
 * second moment about the Monte-Carlo mean (divisor S) is taken, the same
 * divisor as the mean itself. */
int oracle_rank_spread(const double *samples, int S, int N, double *out_mean, double *out_sd) {
    if (!samples || !out_mean || !out_sd || S < 1 || N < 1) return ORACLE_EINVAL;
    double *srt = (double *)malloc(sizeof(double) * (size_t)S * N);
    if (!srt) return ORACLE_EINVAL;
    memcpy(srt, samples, sizeof(double) * (size_t)S * N);
    for (int k = 0; k < S; ++k) qsort(srt + (size_t)k * N, N, sizeof(double), dbl_cmp);
    for (int c = 0; c < N; ++c) {
        double sum = 0.0;
        for (int k = 0; k < S; ++k) sum += srt[(size_t)k * N + c];
        double mean = sum / (double)S, dev = 0.0;
        for (int k = 0; k < S; ++k) {
            double d = srt[(size_t)k * N + c] - mean;
            dev += d * d;
        }
        out_mean[c] = mean;
        out_sd[c] = sqrt(dev / (double)S);
    }
    free(srt);
    return ORACLE_OK;
}
