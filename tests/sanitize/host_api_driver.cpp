// Calls the library's host-side logic (argument checks, size queries, blob parsing, weight
// re-tiling up to the first device call, error paths and their clean-up) with no GPU present.
// Built by tests/test_sanitizers.py with the host code of api.hip and cutoff_select.hip under
// -fsanitize=address,undefined; the run must end with status 0 and no sanitizer report.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "cutoff_dkf.h"

#define EXPECT(cond)                                                  \
    do {                                                              \
        if (!(cond)) { std::printf("line %d: %s\n", __LINE__, #cond); return 1; } \
    } while (0)

int main() {
    dkf_config cfg{};
    cfg.n_workers = 37; cfg.lag = 4; cfg.z_dim = 9; cfg.hidden = 33; cfg.rnn_dim = 21;
    cfg.mlp_dtype = DKF_DTYPE_F32; cfg.emit_mean_act = 0; cfg.max_samples = 50;
    const size_t bytes = dkf_blob_bytes(&cfg);
    EXPECT(bytes > 32);
    dkf_config bad = cfg;
    bad.lag = 0;
    EXPECT(dkf_blob_bytes(&bad) == 0 && dkf_blob_bytes(nullptr) == 0);
    std::vector<char> blob(bytes, 0);
    const int32_t head[8] = {0x57464B44, 1, cfg.n_workers, cfg.lag, cfg.z_dim, cfg.hidden, cfg.rnn_dim, 0};
    std::memcpy(blob.data(), head, sizeof head);
    float *w = reinterpret_cast<float *>(blob.data() + 32);
    for (size_t i = 0; i < (bytes - 32) / 4; ++i) w[i] = 0.01f * (float)((int)(i % 17) - 8);
    dkf_model *m = reinterpret_cast<dkf_model *>(0x1);
    EXPECT(dkf_load_weights(&cfg, blob.data(), bytes - 4, nullptr, &m) == DKF_EBLOB && m == nullptr);
    EXPECT(dkf_load_weights(&bad, blob.data(), bytes, nullptr, &m) == DKF_EINVAL);
    EXPECT(dkf_load_weights(&cfg, blob.data(), bytes, nullptr, nullptr) == DKF_EINVAL);
    blob[0] ^= 1;
    EXPECT(dkf_load_weights(&cfg, blob.data(), bytes, nullptr, &m) == DKF_EBLOB);
    blob[0] ^= 1;
    dkf_config huge = cfg;
    huge.n_workers = 5000;
    EXPECT(dkf_load_weights(&huge, blob.data(), bytes, nullptr, &m) == DKF_EUNSUPPORTED);
    // with no device the first device call fails: whatever was packed on the host is released again
    for (int dtype = 0; dtype < 2; ++dtype) {
        cfg.mlp_dtype = dtype;
        const int rc = dkf_load_weights(&cfg, blob.data(), bytes, nullptr, &m);
        EXPECT(rc < 0 && m == nullptr);
    }
    EXPECT(cutoff_select_workspace(256, 16) > 0 && cutoff_select_workspace(256, 5000) == 0 &&
           cutoff_select_workspace(0, 16) == 0);
    EXPECT(cutoff_select_static_max_workspace() >= cutoff_select_workspace(8192, 2048));
    EXPECT(dkf_impute_workspace(65, 3) == 256 && cutoff_rank_spread_workspace(1, 1) == 256);
    float x[8] = {};
    int32_t cs[2] = {};
    char ws[512];
    EXPECT(cutoff_select(nullptr, 1, 8, 1, 8, 0.f, nullptr, nullptr, nullptr, nullptr, cs, ws, sizeof ws, nullptr) == DKF_EINVAL);
    EXPECT(cutoff_select(x, 1, 8, 5, 2, 0.f, nullptr, nullptr, nullptr, nullptr, cs, ws, sizeof ws, nullptr) == DKF_EINVAL);
    EXPECT(cutoff_select(x, 1, 8, 1, 8, 0.f, nullptr, nullptr, nullptr, nullptr, cs, ws, 0, nullptr) == DKF_EINVAL);
    EXPECT(cutoff_select_static(x, 0, 8, 1, 8, 0.f, nullptr, nullptr, nullptr, nullptr, cs, nullptr) == DKF_EINVAL);
    EXPECT(cutoff_select_static(x, 8192, 4096, 1, 8, 0.f, nullptr, nullptr, nullptr, nullptr, cs, nullptr) == DKF_EUNSUPPORTED);
    EXPECT(dkf_filter_step(nullptr, x, nullptr) == DKF_EINVAL && dkf_check(nullptr, nullptr) == DKF_EINVAL);
    EXPECT(dkf_decide(nullptr, x, 1, nullptr, nullptr, nullptr, 0, cs, nullptr) == DKF_EINVAL);
    EXPECT(dkf_set_sampler(nullptr, 0) == DKF_EINVAL && dkf_set_exchange_spin_limit(nullptr, 1) == DKF_EINVAL);
    EXPECT(dkf_free(nullptr) == DKF_OK && dkf_decide_samples(nullptr) == nullptr);
    size_t n = 0;
    EXPECT(dkf_get_state(nullptr, nullptr, &n) == DKF_EINVAL && dkf_set_state(nullptr, ws, 4) == DKF_EINVAL);
    for (int code = -9; code <= 3; ++code) EXPECT(dkf_strerror(code) != nullptr && dkf_strerror(code)[0] != 0);
    EXPECT(dkf_timing_enable(0x1FF) == DKF_OK && dkf_timing_enable(0) == DKF_OK);
    int32_t launches = 0;
    double ms = 0.0;
    EXPECT(dkf_timing_read(99, &launches, &ms) == DKF_EINVAL);
    std::puts("host api driver ok");
    return 0;
}
