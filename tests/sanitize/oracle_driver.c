/* Runs every exported routine of the CPU oracle once on small seeded inputs.  Built together with
 * oracle/cutoff_oracle.c under -fsanitize=address,undefined by tests/test_sanitizers.py: the run
 * must finish with status 0 and without a sanitizer report.  Checks nothing numerically (the pins
 * do that); sizes are chosen ragged so that an off-by-one in any loop touches a red zone. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/cutoff_oracle.c"

static uint32_t lcg_state = 12345u;
static double unit(void) {
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (double)(lcg_state >> 8) / 16777216.0;
}
static double gauss(void) { return sqrt(-2.0 * log(unit() + 1e-12)) * cos(6.283185307179586 * unit()); }

int main(void) {
    oracle_config c = {7, 3, 5, 9, 11, 0};
    size_t bytes = oracle_blob_bytes(&c), nf = (bytes - 32) / 4;
    char *blob = (char *)malloc(bytes);
    int32_t head[8] = {0x57464B44, 1, c.n_workers, c.lag, c.z_dim, c.hidden, c.rnn_dim, 0};
    memcpy(blob, head, 32);
    float *w = (float *)(blob + 32);
    for (size_t i = 0; i < nf; ++i) w[i] = (float)(0.3 * gauss());
    oracle_model *m = oracle_load_weights(&c, blob, bytes);
    if (!m) return 2;
    if (oracle_load_weights(&c, blob, bytes - 4)) return 3; /* wrong size is refused */
    const int N = c.n_workers, L = c.lag, Z = c.z_dim, H = c.hidden, R = c.rnn_dim, S = 13;
    double *obs = (double *)malloc(sizeof(double) * N);
    for (int t = 0; t < L + 2; ++t) {
        for (int j = 0; j < N; ++j) obs[j] = 0.5 + unit();
        int rc = oracle_filter_step(m, obs);
        if (rc != (t < L - 1 ? ORACLE_WARMUP : ORACLE_OK)) return 4;
    }
    obs[2] = -1.0;
    if (oracle_filter_step(m, obs) != ORACLE_EBADOBS) return 5;
    float *eq = (float *)malloc(sizeof(float) * L * S * Z), *ez = (float *)malloc(sizeof(float) * S * Z),
          *ex = (float *)malloc(sizeof(float) * S * N);
    for (int i = 0; i < L * S * Z; ++i) eq[i] = (float)gauss();
    for (int i = 0; i < S * Z; ++i) ez[i] = (float)gauss();
    for (int i = 0; i < S * N; ++i) ex[i] = (float)gauss();
    double *hl = (double *)malloc(sizeof(double) * L * R), *hr = (double *)malloc(sizeof(double) * L * R);
    if (oracle_encode_window(m, hl, hr) != ORACLE_OK) return 6;
    double *x = (double *)malloc(sizeof(double) * S * N), *zT = (double *)malloc(sizeof(double) * S * Z),
           *zn = (double *)malloc(sizeof(double) * S * Z), *mean = (double *)malloc(sizeof(double) * S * N),
           *sd = (double *)malloc(sizeof(double) * S * N);
    for (int mode = 0; mode < 2; ++mode) {
        if (oracle_set_mlp_bf16(m, mode) != ORACLE_OK) return 7;
        if (oracle_sample_runtimes(m, S, NULL, 0, eq, ez, ex, x, zT, zn, mean, sd) != ORACLE_OK) return 8;
        int32_t rows[3] = {12, 0, 5};
        if (oracle_sample_runtimes(m, S, rows, 3, eq, ez, ex, x, NULL, NULL, NULL, NULL) != ORACLE_OK) return 9;
        double *gh = (double *)malloc(sizeof(double) * 3 * H), *tz = (double *)malloc(sizeof(double) * 3 * Z * 6);
        if (oracle_transition_terms(m, S, rows, 3, eq, ez, ex, gh, tz, tz + 3 * Z, tz + 6 * Z, tz + 9 * Z, tz + 12 * Z,
                                    tz + 15 * Z) != ORACLE_OK) return 10;
        free(gh); free(tz);
        int32_t cstar = 0;
        if (oracle_predict_cutoff(m, S, eq, ez, ex, 1, N, 0.0, &cstar) < 0 || cstar < 1 || cstar > N) return 11;
    }
    oracle_sample_runtimes(m, S, NULL, 0, eq, ez, ex, x, NULL, NULL, NULL, NULL);
    double *srt = (double *)malloc(sizeof(double) * S * N), *mn = (double *)malloc(sizeof(double) * N),
           *om = (double *)malloc(sizeof(double) * N);
    int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * S * N), cs[1];
    if (oracle_cutoff_select(x, S, N, 2, N - 1, -INFINITY, srt, perm, mn, om, cs) < 0) return 12;
    if (oracle_cutoff_select(x, S, N, 1, N, 0.0, NULL, NULL, NULL, NULL, cs) < 0) return 13;
    float *xf = (float *)malloc(sizeof(float) * S * N);
    for (int i = 0; i < S * N; ++i) xf[i] = (float)x[i];
    if (oracle_cutoff_select_f32(xf, S, N, 1, N, 0.0, srt, perm, mn, om, cs) < 0) return 14;
    double *sdv = (double *)malloc(sizeof(double) * N);
    if (oracle_rank_spread(x, S, N, mn, sdv) < 0) return 15;
    float *xo = (float *)malloc(sizeof(float) * N), *u = (float *)malloc(sizeof(float) * N),
          *full = (float *)malloc(sizeof(float) * N);
    uint8_t *cens = (uint8_t *)malloc(N);
    int32_t *nex = (int32_t *)malloc(sizeof(int32_t) * N);
    for (int j = 0; j < N; ++j) { xo[j] = 1.0f; u[j] = (float)unit() * 0.999f; cens[j] = (uint8_t)(j & 1); }
    if (oracle_impute_censored(xf, S, N, xo, cens, 0.5f, u, full, nex) < 0) return 16;
    if (oracle_impute_censored(xf, S, N, xo, cens, 1e30f, u, full, NULL) < 0) return 17;
    uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6}, out[4];
    oracle_philox4x32_10(ctr, key, out);
    float nb[11];
    oracle_fill_normal(99u, 2u, 11, nb);
    double em[5], eo[5];
    if (oracle_elfving_mean(158, 158, 1.057, 0.393) < 1.0) return 18;
    if (oracle_cutoff_elfving(5, 1.0, 0.2, 1, 5, 0.0, em, eo, cs) < 0) return 19;
    double tr[3 * 4] = {1, 2, 3, 4, 4, 3, 2, 1, 2, 2, 2, 2}, thr[3];
    int32_t cuts[3] = {4, 1, 2};
    if (oracle_trace_throughput(tr, 3, 4, cuts, thr) < 0) return 20;
    oracle_reset(m);
    if (oracle_sample_runtimes(m, S, NULL, 0, eq, ez, ex, x, NULL, NULL, NULL, NULL) != ORACLE_ENOTREADY) return 21;
    (void)oracle_round_bf16(1.0 / 3.0); (void)oracle_scale(m); (void)oracle_num_threads(); oracle_set_threads(2);
    oracle_free(m);
    free(blob); free(obs); free(eq); free(ez); free(ex); free(hl); free(hr); free(x); free(zT); free(zn); free(mean);
    free(sd); free(srt); free(mn); free(om); free(perm); free(xf); free(sdv); free(xo); free(u); free(full); free(cens);
    free(nex);
    puts("oracle driver ok");
    return 0;
}
