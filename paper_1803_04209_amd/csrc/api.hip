// C ABI of libcutoff_dkf.so: model object, host-side window bookkeeping,
// weight re-tiling, stream/graph orchestration.  All arithmetic of the
// predictor runs in the kernels of the other .hip files; this file only moves data and launches them.
#include <chrono>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"

namespace dkf {

// ---- errors -------------------------------------------------------------------
static thread_local hipError_t g_last_hip = hipSuccess;
void set_last_hip_error(hipError_t e) { g_last_hip = e; }

// ---- stage timing ---------------------------------------------------------------
namespace {
constexpr int kMaxRecords = 4096;
struct StageRecords {
    std::vector<hipEvent_t> start, stop;
    int used = 0;
};
std::mutex g_timing_mu;
uint32_t g_timing_mask = 0;
StageRecords g_records[DKF_NUM_STAGES];
thread_local int g_capturing = 0;  // > 0 while a graph is being captured on this thread
}  // namespace

StageTimer::StageTimer(int stage, hipStream_t stream) : slot_(-1), stage_(stage), stream_(stream) {
    if (g_capturing || stage < 0 || stage >= DKF_NUM_STAGES) return;
    std::lock_guard<std::mutex> lock(g_timing_mu);
    if (!(g_timing_mask & (1u << stage))) return;
    StageRecords &r = g_records[stage];
    if (r.used >= kMaxRecords) return;
    if ((int)r.start.size() <= r.used) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return;
        if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
        r.start.push_back(a);
        r.stop.push_back(b);
    }
    slot_ = r.used++;
    (void)hipEventRecord(r.start[slot_], stream_);
}

StageTimer::~StageTimer() {
    if (slot_ < 0) return;
    std::lock_guard<std::mutex> lock(g_timing_mu);
    (void)hipEventRecord(g_records[stage_].stop[slot_], stream_);
}

}  // namespace dkf

using namespace dkf;

// ---- model ------------------------------------------------------------------------
struct dkf_model {
    dkf_config cfg{};
    int N = 0, L = 0, Z = 0, H = 0, R = 0;
    int Np = 0, Zp = 0, Hp = 0, Rp = 0;
    std::vector<void *> dev_allocs;
    std::vector<void *> host_allocs;

    // weights
    const float *w_ih_f = nullptr, *w_ih_b = nullptr, *w_hh_f = nullptr, *w_hh_b = nullptr;
    const float *bias_f = nullptr, *bias_b = nullptr, *z0 = nullptr;
    PackedLayer comb, mu, sig, gate1, gate2, prop1, prop2, lin, tscale;
    PackedLayer emean1, emean2, escale1, escale2;
    bool use_chain = false;  // sizes covered by the register-chained sampler
    const float *chain_guide = nullptr, *chain_stream = nullptr, *chain_bias = nullptr;
    int chain_chunks = 0;
    int sampler = DKF_SAMPLER_AUTO;  // dkf_set_sampler
    bool use_quad = false;   // sizes covered by the four-samples-per-wavefront sampler (small S)
    const float *quad_guide = nullptr, *quad_stream = nullptr, *quad_bias = nullptr;
    int quad_chunks = 0;
    bool use_split = false;  // sizes covered by the sixteen-samples-per-workgroup sampler
    int split_waves = 8;     // wavefronts per workgroup of that sampler: two per SIMD, so that one issues while the other waits
    const float *split_stream = nullptr, *split_bias = nullptr;
    bool use_gchain = false;  // bf16 sizes covered by the register-resident guide/transition kernel
    const float *gc_tiles = nullptr, *gc_bias = nullptr, *gc_mu_w32 = nullptr, *gc_mu_b32 = nullptr;
    float *gc_cmu = nullptr;
    int gc_bias_floats = 0;
    // emission layers and activations in fragment order (egemm.hip), bf16 models with use_gchain
    const float *ef_w[4] = {}, *ef_b[4] = {};  // emean1, emean2, escale1, escale2
    int ef_Hp = 0, ef_Np = 0, ef_samp_tiles = 0;
    float *h1frag = nullptr, *h2frag = nullptr;


    // filter state
    float *d_in = nullptr;  // [Np] observation + Control
    float *proj_f = nullptr, *proj_b = nullptr, *ctx_f = nullptr, *ctx_b = nullptr;
    int32_t *fault = nullptr;   // dev: raised by the multi-workgroup encoder when its bounded wait ran out
    int32_t *xcd_claims = nullptr;  // dev int32[2], see FilterArgs
    bool same_xcd = false;
    int spin_limit = kCoopSpinLimit;
    std::vector<float> window;  // host mirror, ring [L][N]
    int64_t pushes = 0;
    float scale = 0.f;

    // pinned staging for the eager path (ring) and for the graph path (one slot)
    static constexpr int kStagingSlots = 4;
    float *staging[kStagingSlots] = {};
    hipEvent_t staging_done[kStagingSlots] = {};
    bool staging_used[kStagingSlots] = {};
    int staging_next = 0;
    float *staging_graph = nullptr;
    int32_t *cstar_host = nullptr;  // pinned int32[4]: c*, status, then one 64-bit word {ticket | status | c*} of the same decision
    int32_t ticket = 0;             // sequence number of the last decision handed to the GPU
    int32_t filter_seq = 0;         // Control::seq of the last filter step staged

    // workspace
    float *z_next = nullptr, *hid1 = nullptr, *mean = nullptr, *hid2 = nullptr;
    float *samples = nullptr;  // [max_samples][N] used by dkf_decide
    void *cutoff_ws = nullptr;
    size_t cutoff_ws_bytes = 0;
    int32_t *d_cstar = nullptr;
    float *sink = nullptr;  // scratch for masked-off lanes of the sampler
    float *gen_q = nullptr, *gen_z = nullptr, *gen_x = nullptr;  // noise drawn by the library itself

    // captured decision graph
    hipStream_t own_stream = nullptr;
    hipGraph_t graph = nullptr;
    hipGraphExec_t graph_exec = nullptr;
    int graph_S = 0;
    int graph_spin_limit = 0;  // the captured kernels carry the limit of the time of capture
    hipStream_t graph_stream = nullptr;  // stream of the last launch of graph_exec
    bool graph_launched = false;
    const float *graph_eps[3] = {nullptr, nullptr, nullptr};

    size_t in_floats() const { return (size_t)Np + sizeof(Control) / sizeof(float); }
    Control *ctl_dev() const { return reinterpret_cast<Control *>(d_in + Np); }
};

namespace {

int dev_alloc(dkf_model *m, size_t bytes, void **out, bool zero) {
    void *p = nullptr;
    if (bytes == 0) bytes = 256;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
        set_last_hip_error(e);
        return e == hipErrorOutOfMemory ? DKF_ENOMEM : DKF_EHIP;
    }
    m->dev_allocs.push_back(p);
    if (zero) DKF_HIP_TRY(hipMemset(p, 0, bytes));
    *out = p;
    return DKF_OK;
}

int upload(dkf_model *m, const float *src, size_t n, const float **out) {
    void *p = nullptr;
    int rc = dev_alloc(m, n * sizeof(float), &p, false);
    if (rc != DKF_OK) return rc;
    DKF_HIP_TRY(hipMemcpy(p, src, n * sizeof(float), hipMemcpyHostToDevice));
    *out = static_cast<const float *>(p);
    return DKF_OK;
}

// fp32 -> bf16, round to nearest even (the rounding v_cvt_pk_bf16_f32 applies on the device)
uint16_t to_bf16(float f) {
    uint32_t u;
    std::memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Re-tile W[n_out][k_in] (row-major) for the MFMA B operand; see PackedLayer.
int pack_layer(dkf_model *m, const float *w, const float *b, int n_out, int k_in, PackedLayer *out) {
    const bool bf16 = m->cfg.mlp_dtype == DKF_DTYPE_BF16;
    PackedLayer p;
    p.n_out = n_out;
    p.k_in = k_in;
    p.n_blocks = (n_out + 31) / 32;
    p.k_groups = bf16 ? round_up(k_in, 64) / 16 : round_up(k_in, 32) / 8;
    std::vector<float> tiles((size_t)p.n_blocks * p.k_groups * 256, 0.f);  // 64 lanes x 16 bytes per k-group
    uint16_t *half = reinterpret_cast<uint16_t *>(tiles.data());
    const int per_lane = bf16 ? 8 : 4;
    for (int nb = 0; nb < p.n_blocks; ++nb)
        for (int kg = 0; kg < p.k_groups; ++kg)
            for (int lane = 0; lane < 64; ++lane) {
                const int n = nb * 32 + (lane & 31);
                if (n >= n_out) continue;
                const size_t entry = ((size_t)nb * p.k_groups + kg) * 64 + lane;
                for (int j = 0; j < per_lane; ++j) {
                    const int k = kg * 2 * per_lane + (lane >> 5) * per_lane + j;
                    if (k >= k_in) continue;
                    if (bf16) half[entry * 8 + j] = to_bf16(w[(size_t)n * k_in + k]);
                    else tiles[entry * 4 + j] = w[(size_t)n * k_in + k];
                }
            }
    std::vector<float> bias((size_t)p.n_blocks * 32, 0.f);
    for (int n = 0; n < n_out; ++n) bias[n] = b[n];
    int rc = upload(m, tiles.data(), tiles.size(), &p.tiles);
    if (rc != DKF_OK) return rc;
    rc = upload(m, bias.data(), bias.size(), &p.bias);
    if (rc != DKF_OK) return rc;
    *out = p;
    return DKF_OK;
}

// One 16 x 16 weight tile for v_mfma_f32_16x16x4_f32 with the weights as the A operand:
// lane = 16*q + i holds W[ob*16 + i][ib*16 + 4q .. 4q+3] (zero outside the matrix).
void append_tile(std::vector<float> &dst, const float *w, int n_out, int k_in, int ob, int ib) {
    const size_t base = dst.size();
    dst.resize(base + 256, 0.f);
    for (int lane = 0; lane < 64; ++lane) {
        const int n = ob * 16 + (lane & 15);
        if (n >= n_out) continue;
        for (int j = 0; j < 4; ++j) {
            const int k = ib * 16 + (lane >> 4) * 4 + j;
            if (k < k_in) dst[base + lane * 4 + j] = w[(size_t)n * k_in + k];
        }
    }
}

struct RawLayers {
    const float *comb, *mu, *sig, *gate1, *gate2, *prop1, *prop2, *lin, *tscale, *emean1, *emean2, *escale1, *escale2;
    const float *b_comb, *b_mu, *b_sig, *b_gate1, *b_gate2, *b_prop1, *b_prop2, *b_lin, *b_tscale, *b_emean1,
        *b_emean2, *b_escale1, *b_escale2;
};

// The mean I(z) ends in a linear layer, mean = W_I2 h + b_I2, and the scale network's first layer
// is linear in the mean (Sec. 3.1.3, J = MLP_2(I(z))): W_J1 mean + b_J1 = (W_J1 W_I2) h + (W_J1 b_I2 + b_J1).
// That H x H layer, formed once in double precision; w is [H][H] row-major.
void fold_scale_hidden(const RawLayers &r, int H, int N, std::vector<float> &w, std::vector<float> &b) {
    std::vector<double> acc((size_t)H * H, 0.0);
    w.resize((size_t)H * H);
    b.resize(H);
    for (int o = 0; o < H; ++o) {
        double *row = acc.data() + (size_t)o * H;
        double bo = r.b_escale1[o];
        for (int n = 0; n < N; ++n) {
            const double ws = r.escale1[(size_t)o * N + n];
            const float *src = r.emean2 + (size_t)n * H;
            for (int i = 0; i < H; ++i) row[i] += ws * src[i];
            bo += ws * r.b_emean2[n];
        }
        for (int i = 0; i < H; ++i) w[(size_t)o * H + i] = (float)row[i];
        b[o] = (float)bo;
    }
}

// Tile streams of the chained sampler.  Guide: comb [ob group][ib][ob in group], mu [zb][ib], sig [zb][ib].
// Stream: chunks of CH = chain_chunk_tiles(HB) tiles in the order the kernel consumes them, every
// layer padded with zero tiles to whole chunks:
//   gate1 [ib][ob], gate2 [zb][ib], prop1, prop2, lin [ob][ib], tscale, emean1 [ib][ob] (one chunk each);
//   then per group of CH / HB output blocks ob: row ob (ib = 0..HB-1) of the folded H x H layer
//   (fold_scale_hidden);
//   then per group of K2 = CH / (2 HB) 16-worker blocks nb: { emean2 row nb, escale2 row nb
//   (ib = 0..HB-1 each) } for each nb of the group.
// The bias table's escale1 slot holds the folded layer's bias.
int pack_chain(dkf_model *m, const RawLayers &r) {
    const int Z = m->Z, R = m->R, H = m->H, N = m->N;
    const int ZB = (Z + 15) / 16, RB = (R + 15) / 16, HB = (H + 15) / 16, NB = (N + 15) / 16;
    const int CH = chain_chunk_tiles(HB), K2 = CH / (2 * HB);
    std::vector<float> g, s;
    const int GO = RB < 4 ? RB : 4;
    // The kernel evaluates tanh(v) as 1 - 2 / (exp2(2 log2(e) v) + 1): the constant goes into the
    // combiner's matrix and bias here, so the pre-activation arrives as the exponent.
    const double kTanhArg = 2.0 * 1.4426950408889634074;
    std::vector<float> comb_w((size_t)R * Z), comb_b((size_t)R);
    for (size_t i = 0; i < comb_w.size(); ++i) comb_w[i] = (float)(kTanhArg * (double)r.comb[i]);
    for (int i = 0; i < R; ++i) comb_b[i] = (float)(kTanhArg * (double)r.b_comb[i]);
    for (int og = 0; og < RB / GO; ++og)
        for (int ib = 0; ib < ZB; ++ib)
            for (int j = 0; j < GO; ++j) append_tile(g, comb_w.data(), R, Z, og * GO + j, ib);
    for (int zb = 0; zb < ZB; ++zb) for (int ib = 0; ib < RB; ++ib) append_tile(g, r.mu, Z, R, zb, ib);
    for (int zb = 0; zb < ZB; ++zb) for (int ib = 0; ib < ZB; ++ib) append_tile(g, r.sig, Z, Z, zb, ib);
    const size_t chunk = (size_t)CH * 256;
    auto pad = [&] { s.resize((s.size() + chunk - 1) / chunk * chunk, 0.f); };
    auto zeros = [&](int tiles) { s.resize(s.size() + (size_t)tiles * 256, 0.f); };
    auto wide = [&](const float *w) {  // Z -> H
        for (int ib = 0; ib < ZB; ++ib) for (int ob = 0; ob < HB; ++ob) append_tile(s, w, H, Z, ob, ib);
        pad();
    };
    auto narrow = [&](const float *w) {  // H -> Z
        for (int zb = 0; zb < ZB; ++zb) for (int ib = 0; ib < HB; ++ib) append_tile(s, w, Z, H, zb, ib);
        pad();
    };
    auto small = [&](const float *w) {  // Z -> Z
        for (int ob = 0; ob < ZB; ++ob) for (int ib = 0; ib < ZB; ++ib) append_tile(s, w, Z, Z, ob, ib);
        pad();
    };
    wide(r.gate1); narrow(r.gate2); wide(r.prop1); narrow(r.prop2); small(r.lin); small(r.tscale);
    wide(r.emean1);
    std::vector<float> fold_w, fold_b;
    fold_scale_hidden(r, H, N, fold_w, fold_b);
    const int RA = CH / HB;
    for (int c = 0; c < (HB + RA - 1) / RA; ++c)
        for (int u = 0; u < RA; ++u) {
            const int ob = c * RA + u;
            if (ob >= HB) { zeros(HB); continue; }
            for (int ib = 0; ib < HB; ++ib) append_tile(s, fold_w.data(), H, H, ob, ib);
        }
    for (int c = 0; c < (NB + K2 - 1) / K2; ++c)
        for (int u = 0; u < K2; ++u) {
            const int nb = c * K2 + u;
            if (nb >= NB) { zeros(2 * HB); continue; }
            for (int ib = 0; ib < HB; ++ib) append_tile(s, r.emean2, N, H, nb, ib);
            for (int ib = 0; ib < HB; ++ib) append_tile(s, r.escale2, N, H, nb, ib);
        }
    if (s.size() % chunk != 0) return DKF_EINVAL;
    m->chain_chunks = (int)(s.size() / chunk);
    std::vector<float> bt;
    auto add_bias = [&](const float *b, int n, int blocks) {
        const size_t base = bt.size();
        bt.resize(base + (size_t)blocks * 16, 0.f);
        for (int i = 0; i < n; ++i) bt[base + i] = b[i];
    };
    add_bias(comb_b.data(), R, RB); add_bias(r.b_mu, Z, ZB); add_bias(r.b_sig, Z, ZB);
    add_bias(r.b_gate1, H, HB); add_bias(r.b_gate2, Z, ZB); add_bias(r.b_prop1, H, HB); add_bias(r.b_prop2, Z, ZB);
    add_bias(r.b_lin, Z, ZB); add_bias(r.b_tscale, Z, ZB); add_bias(r.b_emean1, H, HB); add_bias(fold_b.data(), H, HB);
    add_bias(r.b_emean2, N, NB); add_bias(r.b_escale2, N, NB);
    bt.resize((size_t)chain_bias_floats(RB * 16, ZB * 16, HB * 16, NB * 16), 0.f);  // whole KiB for the copy into LDS
    int rcb = upload(m, bt.data(), bt.size(), &m->chain_bias);
    if (rcb != DKF_OK) return rcb;
    int rc = upload(m, g.data(), g.size(), &m->chain_guide);
    if (rc != DKF_OK) return rc;
    return upload(m, s.data(), s.size(), &m->chain_stream);
}

// One tile stream per wavefront for the sixteen-samples-per-workgroup sampler (split.hip), in the
// order wavefront w of W = split_waves consumes it (RQ = RB / W, HQ = HB / W, C = 2 HB tiles per chunk, HB for W = 8):
//   guide (wavefronts 0-3, RQ = RB / 4; zeros for the others):  comb [o < RQ][ib] (output block w RQ + o),
//           mu [zb][i < RQ] (input block w RQ + i), sig [zb][ib];
//   head, padded with zero tiles to whole chunks:  gate1 [o < HQ][ib], gate2 [zb][i < HQ], prop1, prop2
//           likewise, lin [ob][ib], tscale [ob][ib], emean1 [o < HQ][ib];
//   the folded H x H layer (fold_scale_hidden):  row w HQ + o (ib < HB) for o < HQ, padded to whole chunks;
//   per own worker block nb = w NBW + u, 2 HB tiles:  emean2 row nb (ib < HB), escale2 row nb (ib < HB);
//   one spare chunk of zeros.
// Biases: the table of the sixteen-per-wavefront kernel.
int pack_split(dkf_model *m, const RawLayers &r) {
    const int Z = m->Z, R = m->R, H = m->H, N = m->N;
    const int ZB = (Z + 15) / 16, RB = (R + 15) / 16, HB = (H + 15) / 16, NB = (N + 15) / 16;
    const int W = m->split_waves;
    const int RQ = RB / 4, HQ = HB / W, C = W == 8 ? HB : 2 * HB, NBW = (NB + W - 1) / W;  // the guide chain runs on wavefronts 0-3
    const int per_wave = split_stream_tiles(Z, R, H, N, W);
    if (per_wave <= 0) return DKF_EINVAL;
    std::vector<float> fold_w, fold_b;
    fold_scale_hidden(r, H, N, fold_w, fold_b);
    std::vector<float> s;
    s.reserve((size_t)W * per_wave * 256);
    for (int w = 0; w < W; ++w) {
        const size_t start = s.size();
        auto pad = [&] {
            const size_t head = start + (size_t)(2 * RQ * ZB + ZB * ZB) * 256, chunk = (size_t)C * 256;
            s.resize(head + (s.size() - head + chunk - 1) / chunk * chunk, 0.f);
        };
        auto zeros = [&](int tiles) { s.resize(s.size() + (size_t)tiles * 256, 0.f); };
        if (w < 4) {
            for (int o = 0; o < RQ; ++o) for (int ib = 0; ib < ZB; ++ib) append_tile(s, r.comb, R, Z, w * RQ + o, ib);
            for (int zb = 0; zb < ZB; ++zb) for (int i = 0; i < RQ; ++i) append_tile(s, r.mu, Z, R, zb, w * RQ + i);
            for (int zb = 0; zb < ZB; ++zb) for (int ib = 0; ib < ZB; ++ib) append_tile(s, r.sig, Z, Z, zb, ib);
        } else {
            zeros(2 * RQ * ZB + ZB * ZB);
        }
        auto wide = [&](const float *wt) { for (int o = 0; o < HQ; ++o) for (int ib = 0; ib < ZB; ++ib) append_tile(s, wt, H, Z, w * HQ + o, ib); };
        auto narrow = [&](const float *wt) { for (int zb = 0; zb < ZB; ++zb) for (int i = 0; i < HQ; ++i) append_tile(s, wt, Z, H, zb, w * HQ + i); };
        auto small = [&](const float *wt) { for (int ob = 0; ob < ZB; ++ob) for (int ib = 0; ib < ZB; ++ib) append_tile(s, wt, Z, Z, ob, ib); };
        wide(r.gate1); narrow(r.gate2); wide(r.prop1); narrow(r.prop2); small(r.lin); small(r.tscale); wide(r.emean1);
        pad();
        for (int o = 0; o < HQ; ++o) for (int ib = 0; ib < HB; ++ib) append_tile(s, fold_w.data(), H, H, w * HQ + o, ib);
        pad();
        for (int u = 0; u < NBW; ++u) {
            const int nb = w * NBW + u;
            if (nb >= NB) { zeros(2 * HB); continue; }
            for (int ib = 0; ib < HB; ++ib) append_tile(s, r.emean2, N, H, nb, ib);
            for (int ib = 0; ib < HB; ++ib) append_tile(s, r.escale2, N, H, nb, ib);
        }
        zeros(C);
        if (s.size() - start != (size_t)per_wave * 256) return DKF_EINVAL;
    }
    std::vector<float> bt;
    auto add_bias = [&](const float *b, int n, int blocks) {
        const size_t base = bt.size();
        bt.resize(base + (size_t)blocks * 16, 0.f);
        for (int i = 0; i < n; ++i) bt[base + i] = b[i];
    };
    add_bias(r.b_comb, R, RB); add_bias(r.b_mu, Z, ZB); add_bias(r.b_sig, Z, ZB);
    add_bias(r.b_gate1, H, HB); add_bias(r.b_gate2, Z, ZB); add_bias(r.b_prop1, H, HB); add_bias(r.b_prop2, Z, ZB);
    add_bias(r.b_lin, Z, ZB); add_bias(r.b_tscale, Z, ZB); add_bias(r.b_emean1, H, HB); add_bias(fold_b.data(), H, HB);
    add_bias(r.b_emean2, N, NB); add_bias(r.b_escale2, N, NB);
    int rc = upload(m, bt.data(), bt.size(), &m->split_bias);
    if (rc == DKF_OK) rc = upload(m, s.data(), s.size(), &m->split_stream);
    return rc;
}

// Tiles and biases of the bf16 guide/transition kernel (layout: GChainArgs).
int pack_gchain(dkf_model *m, const RawLayers &r) {
    const int Z = m->Z, R = m->R, H = m->H;
    const int Q = gchain_q(Z, R, H), HP = 128 * Q, ZT = 2, ZK = 4;
    std::vector<uint16_t> t;
    auto tile = [&](const float *w, int n_out, int k_in, int ob, int ks) {
        const size_t base = t.size();
        t.resize(base + 512, 0);
        for (int lane = 0; lane < 64; ++lane)
            for (int j = 0; j < 8; ++j) {
                const int row = 32 * ob + (lane & 31), k = 16 * ks + 8 * (j >> 2) + 4 * (lane >> 5) + (j & 3);
                if (row < n_out && k < k_in) t[base + lane * 8 + j] = to_bf16(w[(size_t)row * k_in + k]);
            }
    };
    auto wide = [&](const float *w, int n_out) {  // Z -> n_out
        for (int wv = 0; wv < 4; ++wv) for (int ob = 0; ob < Q; ++ob) for (int ks = 0; ks < ZK; ++ks) tile(w, n_out, Z, wv * Q + ob, ks);
    };
    auto narrow = [&](const float *w, int k_in) {  // k_in -> Z
        for (int wv = 0; wv < 4; ++wv) for (int nb = 0; nb < ZT; ++nb) for (int ks = 0; ks < 2 * Q; ++ks) tile(w, Z, k_in, nb, 2 * wv * Q + ks);
    };
    auto small = [&](const float *w) {
        for (int nb = 0; nb < ZT; ++nb) for (int ks = 0; ks < ZK; ++ks) tile(w, Z, Z, nb, ks);
    };
    wide(r.comb, R); narrow(r.mu, R); small(r.sig);
    wide(r.gate1, H); narrow(r.gate2, H); wide(r.prop1, H); narrow(r.prop2, H); small(r.lin); small(r.tscale);
    wide(r.emean1, H);
    std::vector<float> bt;
    auto add_bias = [&](const float *b, int n, int padded) {
        const size_t base = bt.size();
        bt.resize(base + (size_t)padded, 0.f);
        for (int i = 0; i < n; ++i) bt[base + i] = b[i];
    };
    add_bias(r.b_comb, R, HP); add_bias(r.b_sig, Z, 64); add_bias(r.b_gate1, H, HP); add_bias(r.b_gate2, Z, 64);
    add_bias(r.b_prop1, H, HP); add_bias(r.b_prop2, Z, 64); add_bias(r.b_lin, Z, 64); add_bias(r.b_tscale, Z, 64);
    add_bias(r.b_emean1, H, HP);
    m->gc_bias_floats = (int)bt.size();
    std::vector<float> as_floats(t.size() / 2);
    std::memcpy(as_floats.data(), t.data(), t.size() * sizeof(uint16_t));
    int rc = upload(m, as_floats.data(), as_floats.size(), &m->gc_tiles);
    if (rc == DKF_OK) rc = upload(m, bt.data(), bt.size(), &m->gc_bias);
    if (rc == DKF_OK) rc = upload(m, r.mu, (size_t)Z * R, &m->gc_mu_w32);
    if (rc == DKF_OK) rc = upload(m, r.b_mu, (size_t)Z, &m->gc_mu_b32);
    void *q = nullptr;
    if (rc == DKF_OK) rc = dev_alloc(m, (size_t)m->L * 64 * sizeof(float), &q, true);
    m->gc_cmu = static_cast<float *>(q);
    return rc;
}

// One dense layer as weight fragments [m_pad / 32][k_pad / 16] (same tile format as pack_gchain) + padded bias.
int pack_frag_layer(dkf_model *m, const float *w, const float *b, int n_out, int k_in, int m_pad, int k_pad,
                    const float **tiles_out, const float **bias_out) {
    std::vector<uint16_t> t((size_t)(m_pad / 32) * (k_pad / 16) * 512, 0);
    for (int ob = 0; ob < m_pad / 32; ++ob)
        for (int ks = 0; ks < k_pad / 16; ++ks) {
            uint16_t *dst = t.data() + ((size_t)ob * (k_pad / 16) + ks) * 512;
            for (int lane = 0; lane < 64; ++lane)
                for (int j = 0; j < 8; ++j) {
                    const int row = 32 * ob + (lane & 31), k = 16 * ks + 8 * (j >> 2) + 4 * (lane >> 5) + (j & 3);
                    if (row < n_out && k < k_in) dst[lane * 8 + j] = to_bf16(w[(size_t)row * k_in + k]);
                }
        }
    std::vector<float> as_floats(t.size() / 2);
    std::memcpy(as_floats.data(), t.data(), t.size() * sizeof(uint16_t));
    std::vector<float> bias(m_pad, 0.f);
    for (int i = 0; i < n_out; ++i) bias[i] = b[i];
    int rc = upload(m, as_floats.data(), as_floats.size(), tiles_out);
    if (rc == DKF_OK) rc = upload(m, bias.data(), bias.size(), bias_out);
    return rc;
}

// The bf16 emission (egemm.hip), with the scale network's first layer folded (fold_scale_hidden).
int pack_emission_frags(dkf_model *m, const RawLayers &r) {
    const int H = m->H, N = m->N;
    const int Hp = round_up(H, 128), Np = round_up(N, 128);
    m->ef_Hp = Hp; m->ef_Np = Np;
    m->ef_samp_tiles = (m->cfg.max_samples + 255) / 256;
    std::vector<float> fold_w, fold_bf;
    fold_scale_hidden(r, H, N, fold_w, fold_bf);
    // (the mean's first layer is part of the guide/transition kernel's tiles: pack_gchain)
    int rc = pack_frag_layer(m, r.emean2, r.b_emean2, N, H, Np, Hp, &m->ef_w[1], &m->ef_b[1]);
    if (rc == DKF_OK) rc = pack_frag_layer(m, fold_w.data(), fold_bf.data(), H, H, Hp, Hp, &m->ef_w[2], &m->ef_b[2]);
    if (rc == DKF_OK) rc = pack_frag_layer(m, r.escale2, r.b_escale2, N, H, Np, Hp, &m->ef_w[3], &m->ef_b[3]);
    const size_t blocks = (size_t)m->ef_samp_tiles * 8;  // 32-sample blocks
    void *q = nullptr;
    if (rc == DKF_OK) rc = dev_alloc(m, blocks * (Hp / 16) * 1024, &q, true);
    m->h1frag = static_cast<float *>(q);
    if (rc == DKF_OK) rc = dev_alloc(m, blocks * (Hp / 16) * 1024, &q, true);
    m->h2frag = static_cast<float *>(q);
    return rc;
}

// The emission on fragments: the scale's hidden layer (folded) and both output layers with the
// draw; the mean's hidden layer comes, as fragments, from the guide/transition kernel.
int enqueue_emission_frags(dkf_model *m, int S, const float *eps_x, float *out_samples, const dkf_stage_outputs *st,
                           hipStream_t stream) {
    FragGemmArgs e{};
    e.S = S; e.N = m->N; e.ctl = m->ctl_dev();
    const int Hp = m->ef_Hp, Np = m->ef_Np;
    e.tile = 2; e.samp_tiles = (S + 255) / 256;
    int rc;
    e.feat_tiles = Hp / 64; e.out_k_steps = Hp / 16;
    e.wfrag = m->ef_w[2]; e.bias = m->ef_b[2]; e.xfrag = m->h1frag; e.k_steps = Hp / 16;
    e.epilogue = kFragRelu; e.out_frag = m->h2frag;
    if ((rc = launch_frag_gemm(e, kStageEmitScaleHidden, stream)) != DKF_OK) return rc;
    e.wfrag = m->ef_w[3]; e.bias = m->ef_b[3]; e.xfrag = m->h2frag;
    e.wfrag2 = m->ef_w[1]; e.bias2 = m->ef_b[1]; e.xfrag2 = m->h1frag;
    e.feat_tiles = Np / 64;
    e.epilogue = kFragDraw; e.out_frag = nullptr; e.out_k_steps = 0;
    e.eps_x = eps_x; e.out_samples = out_samples;
    e.out_mean_dbg = st ? st->emit_mean : nullptr;
    e.out_sd_dbg = st ? st->emit_sd : nullptr;
    return launch_frag_gemm(e, kStageEmitScaleDraw, stream);
}

size_t blob_floats(const dkf_config *c) {
    const size_t N = c->n_workers, Z = c->z_dim, H = c->hidden, R = c->rnn_dim;
    const size_t rnn = 2 * (R * N + R + R * R + R);
    const size_t guide = R * Z + R + Z * R + Z + Z * Z + Z + Z;
    const size_t trans = 2 * (H * Z + H + Z * H + Z) + 2 * (Z * Z + Z);
    const size_t emit = H * Z + H + N * H + N + H * N + H + N * H + N;
    return rnn + guide + trans + emit;
}

bool config_ok(const dkf_config *c) {
    return c && c->n_workers >= 1 && c->lag >= 1 && c->z_dim >= 1 && c->hidden >= 1 && c->rnn_dim >= 1 &&
           c->max_samples >= 1 && (c->mlp_dtype == DKF_DTYPE_F32 || c->mlp_dtype == DKF_DTYPE_BF16) &&
           (c->emit_mean_act == 0 || c->emit_mean_act == 1);
}

// Tile streams of the four-samples-per-wavefront sampler (quad.hip).  A tile is 64 lanes x 4
// floats; entry e of lane l is the B operand of the tile's e-th matrix instruction:
//   wide layer, narrow input, tile (zq, kg):    W[64 og + l][16 zq + 4 kg + e]
//   wide layer, wide input, tile (og, ig, b):   W[64 og + l][64 ig + 4 b + e]
//   narrow layer, wide input, tile (zq, ig, q): W[16 zq + (l & 15)][64 ig + 16 (l >> 4) + 4 q + e]
//   narrow layer, narrow input, tile (zo, zi):  W[16 zo + (l & 15)][16 zi + 4 (l >> 4) + e]
// (zero outside the matrix).  Guide: comb [zq][kg][og], mu [zq][ig][q], sig [zo][zi].  Stream:
// the transition layers and the emission's first layer at the positions of quad_plan(); then per
// 64-worker group og the mean's second layer [ig][b] followed by that group's columns of the
// scale network's first layer [b][hg]; then per group the scale network's second layer [ig][b].
int pack_quad(dkf_model *m, const RawLayers &r) {
    const int Z = m->Z, R = m->R, H = m->H, N = m->N;
    const int ZQ = (Z + 15) / 16, RG = (R + 63) / 64, HG = (H + 63) / 64, NG = (N + 63) / 64;
    const int CH = kQuadChunkTiles;
    auto tile = [](std::vector<float> &dst, size_t at, const float *w, int n_out, int k_in, auto &&row, auto &&col) {
        if (dst.size() < (at + 1) * 256) dst.resize((at + 1) * 256, 0.f);
        for (int lane = 0; lane < 64; ++lane)
            for (int e = 0; e < 4; ++e) {
                const int n = row(lane), k = col(lane, e);
                if (n < n_out && k < k_in) dst[at * 256 + lane * 4 + e] = w[(size_t)n * k_in + k];
            }
    };
    auto wide_q = [&](std::vector<float> &dst, size_t at, const float *w, int n_out, int k_in, int groups) {  // [zq][kg][og]
        for (int zq = 0; zq < ZQ; ++zq) for (int kg = 0; kg < 4; ++kg) for (int og = 0; og < groups; ++og)
            tile(dst, at++, w, n_out, k_in, [&](int l) { return 64 * og + l; },
                 [&](int, int e) { return 16 * zq + 4 * kg + e; });
    };
    auto narrow_a = [&](std::vector<float> &dst, size_t at, const float *w, int n_out, int k_in, int groups) {  // [zq][ig][q]
        for (int zq = 0; zq < ZQ; ++zq) for (int ig = 0; ig < groups; ++ig) for (int q = 0; q < 4; ++q)
            tile(dst, at++, w, n_out, k_in, [&](int l) { return 16 * zq + (l & 15); },
                 [&](int l, int e) { return 64 * ig + 16 * (l >> 4) + 4 * q + e; });
    };
    auto narrow_q = [&](std::vector<float> &dst, size_t at, const float *w) {  // [zo][zi], Z x Z
        for (int zo = 0; zo < ZQ; ++zo) for (int zi = 0; zi < ZQ; ++zi)
            tile(dst, at++, w, Z, Z, [&](int l) { return 16 * zo + (l & 15); },
                 [&](int l, int e) { return 16 * zi + 4 * (l >> 4) + e; });
    };
    std::vector<float> g, s;
    wide_q(g, 0, r.comb, R, Z, RG);
    narrow_a(g, (size_t)4 * ZQ * RG, r.mu, Z, R, RG);
    narrow_q(g, (size_t)8 * ZQ * RG, r.sig);
    const QuadPlan plan = quad_plan(ZQ, HG);
    s.resize((size_t)plan.head_chunks * CH * 256, 0.f);
    wide_q(s, plan.gate1, r.gate1, H, Z, HG);
    wide_q(s, plan.prop1, r.prop1, H, Z, HG);
    narrow_q(s, plan.lin, r.lin);
    narrow_a(s, plan.gate2, r.gate2, Z, H, HG);
    narrow_a(s, plan.prop2, r.prop2, Z, H, HG);
    narrow_q(s, plan.tscale, r.tscale);
    wide_q(s, plan.emean1, r.emean1, H, Z, HG);
    size_t at = (size_t)plan.head_chunks * CH;
    for (int og = 0; og < NG; ++og) {
        for (int t = 0; t < 16 * HG; ++t) {  // mean, second layer: tile (ig, b)
            const int ig = t / 16, b = t % 16;
            tile(s, at++, r.emean2, N, H, [&](int l) { return 64 * og + l; }, [&](int, int e) { return 64 * ig + 4 * b + e; });
        }
        for (int t = 0; t < 16 * HG; ++t) {  // scale network, first layer, input columns of group og: tile (b, hg)
            const int b = t / HG, hg = t % HG;
            tile(s, at++, r.escale1, H, N, [&](int l) { return 64 * hg + l; }, [&](int, int e) { return 64 * og + 4 * b + e; });
        }
    }
    for (int og = 0; og < NG; ++og) {
        for (int t = 0; t < 16 * HG; ++t) {
            const int ig = t / 16, b = t % 16;
            tile(s, at++, r.escale2, N, H, [&](int l) { return 64 * og + l; }, [&](int, int e) { return 64 * ig + 4 * b + e; });
        }
        at = (at + CH - 1) / CH * CH;  // a group starts on a chunk
    }
    s.resize(at * 256, 0.f);
    m->quad_chunks = (int)(at / CH);
    std::vector<float> bt;
    auto add_bias = [&](const float *b, int n, int padded) {
        const size_t base = bt.size();
        bt.resize(base + (size_t)padded, 0.f);
        for (int i = 0; i < n; ++i) bt[base + i] = b[i];
    };
    const int Z16 = 16 * ZQ, R64 = 64 * RG, H64 = 64 * HG, N64 = 64 * NG;
    add_bias(r.b_comb, R, R64); add_bias(r.b_mu, Z, Z16); add_bias(r.b_sig, Z, Z16);
    add_bias(r.b_gate1, H, H64); add_bias(r.b_gate2, Z, Z16); add_bias(r.b_prop1, H, H64); add_bias(r.b_prop2, Z, Z16);
    add_bias(r.b_lin, Z, Z16); add_bias(r.b_tscale, Z, Z16); add_bias(r.b_emean1, H, H64); add_bias(r.b_escale1, H, H64);
    add_bias(r.b_emean2, N, N64); add_bias(r.b_escale2, N, N64);
    int rc = upload(m, bt.data(), bt.size(), &m->quad_bias);
    if (rc == DKF_OK) rc = upload(m, g.data(), g.size(), &m->quad_guide);
    if (rc == DKF_OK) rc = upload(m, s.data(), s.size(), &m->quad_stream);
    return rc;
}

// `input`: where the step's observation + control block is read from (pinned host staging or d_in)
FilterArgs filter_args(const dkf_model *m, const float *input) {
    FilterArgs a;
    a.input = input;
    a.mirror = m->d_in;
    a.ctl = m->ctl_dev();
    a.proj_f = m->proj_f; a.proj_b = m->proj_b;
    a.ctx_f = m->ctx_f; a.ctx_b = m->ctx_b;
    a.w_ih_f = m->w_ih_f; a.w_ih_b = m->w_ih_b;
    a.w_hh_f = m->w_hh_f; a.w_hh_b = m->w_hh_b;
    a.bias_f = m->bias_f; a.bias_b = m->bias_b;
    a.N = m->N; a.Np = m->Np; a.L = m->L; a.R = m->R; a.Rp = m->Rp;
    a.fault = m->fault;
    a.proj_flags = m->fault + 32;
    a.spin_limit = m->spin_limit;
    a.xcd_claims = m->xcd_claims;
    a.same_xcd = m->same_xcd;
    a.encode = true;
    return a;
}

// Host bookkeeping of one push: validates, updates the window mirror and the
// normaliser, and fills `dst` (pinned) with the observation and its Control.
// Control::seq of the next filter step: counts up for as long as the model lives (dkf_reset does
// not rewind it), skipping zero, so a value is never seen twice by the device
int32_t next_filter_seq(dkf_model *m) {
    m->filter_seq = m->filter_seq == INT32_MAX ? 1 : m->filter_seq + 1;
    return m->filter_seq;
}

int stage_observation(dkf_model *m, const float *x_obs, uint64_t seed, float *dst) {
    const int N = m->N, L = m->L;
    for (int j = 0; j < N; ++j)
        if (!std::isfinite(x_obs[j]) || !(x_obs[j] > 0.f)) return DKF_EBADOBS;
    const int slot = (int)(m->pushes % L);
    std::memcpy(&m->window[(size_t)slot * N], x_obs, sizeof(float) * N);
    m->pushes++;
    const int count = m->pushes < L ? (int)m->pushes : L;
    if (m->pushes == L) {
        // normaliser: twice the mean of the first complete window, fixed from here on
        double sum = 0.0;
        for (size_t i = 0; i < (size_t)L * N; ++i) sum += (double)m->window[i];
        m->scale = (float)(2.0 * sum / ((double)L * N));
    }
    std::memcpy(dst, x_obs, sizeof(float) * N);
    for (int j = N; j < m->Np; ++j) dst[j] = 0.f;
    Control c;
    c.slot = slot;
    c.count = count;
    c.oldest = count < L ? 0 : (slot + 1) % L;
    c.ticket = 0;
    c.scale = m->scale;
    c.inv_scale = m->scale > 0.f ? 1.0f / m->scale : 0.f;
    c.seed_lo = (uint32_t)seed;
    c.seed_hi = (uint32_t)(seed >> 32);
    c.seq = next_filter_seq(m);
    std::memcpy(dst + m->Np, &c, sizeof c);
    return count < L ? DKF_WARMUP : DKF_OK;
}

int copy_ctx(dkf_model *m, float *dst, hipStream_t stream);

// Host polls of the decision's ticket before falling back to a stream synchronisation (a few
// hundred milliseconds: far beyond any decision this library takes).
constexpr long kTicketSpins = 50L * 1000 * 1000;

// Up to this many samples the four-per-wavefront sampler is used where both are available (at
// 16 per wavefront, 16384 samples are what fills every SIMD of the chip once).
constexpr int kQuadMaxSamples = 8192;
// Up to this many samples (one workgroup of sixteen per compute unit) the sampler that splits
// every layer over a workgroup's wavefronts has the shortest critical path.
constexpr int kSplitMaxSamples = 4096;

// The kernel family a call with S samples launches: one of the fused fp32 kernels, or
// DKF_SAMPLER_STAGED for everything that runs as several kernels.
int sampler_for(const dkf_model *m, int S) {
    if (m->sampler == DKF_SAMPLER_STAGED || !(m->use_chain || m->use_quad || m->use_split)) return DKF_SAMPLER_STAGED;
    if (m->sampler != DKF_SAMPLER_AUTO) return m->sampler;
    // few samples: sixteen per workgroup or four per wavefront, so that they still spread over the whole chip
    if (m->use_split && (S <= kSplitMaxSamples || (!m->use_chain && !m->use_quad))) return DKF_SAMPLER_SPLIT;
    if (m->use_quad && (S <= kQuadMaxSamples || !m->use_chain)) return DKF_SAMPLER_WAVE4;
    return DKF_SAMPLER_WAVE16;
}

int enqueue_chain(dkf_model *m, int S, const float *eps_q, const float *eps_z, const float *eps_x,
                  float *out_samples, const dkf_stage_outputs *st, hipStream_t stream, float *rank_partial = nullptr,
                  uint32_t *rank_done = nullptr) {
    const int variant = sampler_for(m, S);
    const bool split = variant == DKF_SAMPLER_SPLIT, quad = variant == DKF_SAMPLER_WAVE4;
    ChainArgs c{};
    c.ctl = m->ctl_dev();
    c.ctx_f = m->ctx_f; c.ctx_b = m->ctx_b; c.Rp = m->Rp;
    if (split) {
        c.stream_tiles = m->split_stream; c.bias_table = m->split_bias; c.split_waves = m->split_waves;
    } else if (quad) {
        c.guide_tiles = m->quad_guide; c.stream_tiles = m->quad_stream; c.stream_chunks = m->quad_chunks;
        c.bias_table = m->quad_bias;
    } else {
        c.guide_tiles = m->chain_guide; c.stream_tiles = m->chain_stream; c.stream_chunks = m->chain_chunks;
        c.bias_table = m->chain_bias;
    }
    c.z0 = m->z0;
    c.eps_q = eps_q; c.eps_z = eps_z; c.eps_x = eps_x;
    c.mean = m->mean; c.ld_mean = m->Np;
    c.out_samples = out_samples;
    c.sink = m->sink;
    c.z_last = st ? st->z_last : nullptr;
    c.z_next_dbg = st ? st->z_next : nullptr;
    c.out_mean_dbg = st ? st->emit_mean : nullptr;
    c.out_sd_dbg = st ? st->emit_sd : nullptr;
    c.S = S; c.L = m->L; c.Z = m->Z; c.R = m->R; c.H = m->H; c.N = m->N; c.NB = (m->N + 15) / 16;
    c.emit_mean_act = m->cfg.emit_mean_act;
    if (rank_partial && !split) return DKF_EINVAL;
    c.rank_partial = rank_partial; c.rank_done = rank_done;
    const int rc = split ? launch_split(c, stream) : quad ? launch_quad(c, stream) : launch_chain(c, stream);
    if (rc != DKF_OK) return rc;
    if (st && st->ctx) return copy_ctx(m, st->ctx, stream);
    return DKF_OK;
}

// Draw the three noise tensors for S samples into the model's own buffers.
int enqueue_noise(dkf_model *m, int S, const Control *ctl, uint64_t seed, hipStream_t stream) {
    return launch_fill_normal3(m->gen_q, (size_t)m->L * S * m->Z, m->gen_z, (size_t)S * m->Z, m->gen_x,
                               (size_t)S * m->N, ctl, seed, stream);
}

// Whether the sampler a decision with S samples launches also sorts the rows it draws (then the
// decision has no row-sort launch): the eight-wavefront split sampler at the widths it is built for.
bool sampler_sorts_rows(const dkf_model *m, int S) {
    return sampler_for(m, S) == DKF_SAMPLER_SPLIT &&
           split_sorts_rows(m->Z, m->R, m->H, m->L, m->N, S, m->split_waves) && S / 16 <= cutoff_rank_sum_rows(S, m->N);
}

int enqueue_sample(dkf_model *m, int S, const float *eps_q, const float *eps_z, const float *eps_x,
                   float *out_samples, const dkf_stage_outputs *st, hipStream_t stream, float *rank_partial = nullptr,
                   uint32_t *rank_done = nullptr) {
    if (sampler_for(m, S) != DKF_SAMPLER_STAGED)
        return enqueue_chain(m, S, eps_q, eps_z, eps_x, out_samples, st, stream, rank_partial, rank_done);
    if (rank_partial) return DKF_EINVAL;
    int rc = DKF_EUNSUPPORTED;
    if (m->sampler != DKF_SAMPLER_STAGED && m->use_gchain) {
        GChainArgs c{};
        c.ctl = m->ctl_dev();
        c.ctx_f = m->ctx_f; c.ctx_b = m->ctx_b; c.Rp = m->Rp;
        c.tiles = m->gc_tiles; c.bias_table = m->gc_bias; c.bias_floats = m->gc_bias_floats;
        c.mu_w32 = m->gc_mu_w32; c.mu_b32 = m->gc_mu_b32; c.cmu = m->gc_cmu;
        c.z0 = m->z0;
        c.eps_q = eps_q; c.eps_z = eps_z;
        c.z_last = st ? st->z_last : nullptr;
        c.z_next_dbg = st ? st->z_next : nullptr;
        c.z_next = nullptr;
        c.h1frag = m->h1frag; c.h1_k_steps = m->ef_Hp / 16; c.emit_mean_act = m->cfg.emit_mean_act;
        c.S = S; c.L = m->L; c.Z = m->Z; c.Zp = m->Zp; c.R = m->R; c.H = m->H;
        const bool aligned = ((reinterpret_cast<uintptr_t>(eps_x) | reinterpret_cast<uintptr_t>(out_samples) |
                               (st ? reinterpret_cast<uintptr_t>(st->emit_mean) | reinterpret_cast<uintptr_t>(st->emit_sd) : 0)) & 15) == 0;
        if (aligned) rc = launch_gchain(c, stream);
        if (rc == DKF_OK) {
            rc = enqueue_emission_frags(m, S, eps_x, out_samples, st, stream);
            if (rc != DKF_OK) return rc;
            if (st && st->ctx) return copy_ctx(m, st->ctx, stream);
            return DKF_OK;
        }
        if (rc != DKF_EUNSUPPORTED && rc != DKF_EINVAL) return rc;
    }
    if (rc != DKF_OK) {  // sizes (or caller buffers not 16-byte aligned) the register-resident kernel does not take
        GuideArgs g;
        g.ctl = m->ctl_dev();
        g.ctx_f = m->ctx_f; g.ctx_b = m->ctx_b;
        g.comb = m->comb; g.mu = m->mu; g.sig = m->sig; g.z0 = m->z0;
        g.gate1 = m->gate1; g.prop1 = m->prop1; g.gate2 = m->gate2; g.prop2 = m->prop2;
        g.lin = m->lin; g.tscale = m->tscale;
        g.eps_q = eps_q; g.eps_z = eps_z;
        g.z_last = st ? st->z_last : nullptr;
        g.z_next_dbg = st ? st->z_next : nullptr;
        g.z_next = m->z_next;
        g.S = S; g.L = m->L; g.Z = m->Z; g.Zp = m->Zp; g.R = m->R; g.Rp = m->Rp; g.H = m->H; g.Hp = m->Hp;
        g.bf16 = m->cfg.mlp_dtype == DKF_DTYPE_BF16;
        rc = launch_guide(g, stream);
        if (rc != DKF_OK) return rc;
    }

    GemmArgs e{};
    e.S = S; e.N = m->N; e.ctl = m->ctl_dev();
    e.bf16 = m->cfg.mlp_dtype == DKF_DTYPE_BF16;
    // hidden layer of the mean
    e.A = m->z_next; e.lda = m->Zp; e.layer = m->emean1;
    e.epilogue = m->cfg.emit_mean_act ? kEpiBiasRelu : kEpiBias;
    e.out = m->hid1; e.ldo = m->Hp;
    if ((rc = launch_gemm(e, kStageEmitHidden, stream)) != DKF_OK) return rc;
    // mean
    e.A = m->hid1; e.lda = m->Hp; e.layer = m->emean2; e.epilogue = kEpiBias; e.out = m->mean; e.ldo = m->Np;
    if ((rc = launch_gemm(e, kStageEmitMean, stream)) != DKF_OK) return rc;
    // hidden layer of the scale, fed by the mean
    e.A = m->mean; e.lda = m->Np; e.layer = m->escale1; e.epilogue = kEpiBiasRelu; e.out = m->hid2; e.ldo = m->Hp;
    if ((rc = launch_gemm(e, kStageEmitScaleHidden, stream)) != DKF_OK) return rc;
    // scale, draw, back to seconds
    e.A = m->hid2; e.lda = m->Hp; e.layer = m->escale2; e.epilogue = kEpiScaleDraw; e.out = nullptr; e.ldo = 0;
    e.mean = m->mean; e.ld_mean = m->Np; e.eps_x = eps_x; e.out_samples = out_samples;
    e.out_mean_dbg = st ? st->emit_mean : nullptr;
    e.out_sd_dbg = st ? st->emit_sd : nullptr;
    if ((rc = launch_gemm(e, kStageEmitScaleDraw, stream)) != DKF_OK) return rc;

    if (st && st->ctx) return copy_ctx(m, st->ctx, stream);
    return DKF_OK;
}

// h_left + h_right per window position into a caller buffer [L][R]; inspection only
// (synchronises the stream and goes through the host).
int copy_ctx(dkf_model *m, float *dst, hipStream_t stream) {
    std::vector<float> f((size_t)m->L * m->Rp), b((size_t)m->L * m->Rp), c((size_t)m->L * m->R);
    DKF_HIP_TRY(hipStreamSynchronize(stream));
    DKF_HIP_TRY(hipMemcpy(f.data(), m->ctx_f, f.size() * 4, hipMemcpyDeviceToHost));
    DKF_HIP_TRY(hipMemcpy(b.data(), m->ctx_b, b.size() * 4, hipMemcpyDeviceToHost));
    for (int t = 0; t < m->L; ++t)
        for (int r = 0; r < m->R; ++r) c[(size_t)t * m->R + r] = f[(size_t)t * m->Rp + r] + b[(size_t)t * m->Rp + r];
    DKF_HIP_TRY(hipMemcpy(dst, c.data(), c.size() * 4, hipMemcpyHostToDevice));
    return DKF_OK;
}

// The previous launch may still count as in flight for the runtime (a decision returns as soon as
// its ticket lands in host memory): wait for the stream it ran on before destroying the executable.
void drop_graph(dkf_model *m) {
    if (m->graph_exec && m->graph_launched) (void)hipStreamSynchronize(m->graph_stream);
    m->graph_launched = false;
    if (m->graph_exec) { (void)hipGraphExecDestroy(m->graph_exec); m->graph_exec = nullptr; }
    if (m->graph) { (void)hipGraphDestroy(m->graph); m->graph = nullptr; }
    m->graph_S = 0;
}

}  // namespace

// ---- exported functions ----------------------------------------------------------------
extern "C" {

const char *dkf_strerror(int code) {
    switch (code) {
        case DKF_OK: return "ok";
        case DKF_WARMUP: return "warming up: fewer than L observations";
        case CUTOFF_NO_ELIGIBLE: return "no eligible cutoff; c_max returned";
        case DKF_EINVAL: return "invalid argument";
        case DKF_ENOTREADY: return "window not full";
        case DKF_EBADOBS: return "observation not finite or not positive";
        case DKF_EHIP: return "HIP runtime error";
        case DKF_ENOMEM: return "out of memory";
        case DKF_EBLOB: return "weight blob does not match the configuration";
        case DKF_EUNSUPPORTED: return "size or mode not supported";
        case DKF_ESTALLED: return "filter state exchange gave up: no valid encoding";
        default: return "unknown code";
    }
}

int dkf_last_hip_error(void) { return (int)g_last_hip; }

size_t dkf_blob_bytes(const dkf_config *cfg) {
    if (!config_ok(cfg)) return 0;
    return 32 + 4 * blob_floats(cfg);
}

int dkf_free(dkf_model *m) {
    if (!m) return DKF_OK;
    (void)hipDeviceSynchronize();
    drop_graph(m);
    if (m->own_stream) (void)hipStreamDestroy(m->own_stream);
    for (int i = 0; i < dkf_model::kStagingSlots; ++i)
        if (m->staging_done[i]) (void)hipEventDestroy(m->staging_done[i]);
    for (void *p : m->dev_allocs) (void)hipFree(p);
    for (void *p : m->host_allocs) (void)hipHostFree(p);
    delete m;
    return DKF_OK;
}

int dkf_load_weights(const dkf_config *cfg, const void *blob, size_t blob_bytes, void *stream, dkf_model **out) {
    if (!out) return DKF_EINVAL;
    *out = nullptr;
    if (!config_ok(cfg) || !blob) return DKF_EINVAL;
    if (cfg->n_workers > 4096 || cfg->z_dim > 1024 || cfg->hidden > 1024 || cfg->rnn_dim > 1024 || cfg->lag > 256)
        return DKF_EUNSUPPORTED;
    if (blob_bytes != dkf_blob_bytes(cfg)) return DKF_EBLOB;
    int32_t head[8];
    std::memcpy(head, blob, sizeof head);
    if (head[0] != 0x57464B44 || head[1] != 1 || head[2] != cfg->n_workers || head[3] != cfg->lag ||
        head[4] != cfg->z_dim || head[5] != cfg->hidden || head[6] != cfg->rnn_dim)
        return DKF_EBLOB;

    dkf_model *m = new (std::nothrow) dkf_model();
    if (!m) return DKF_ENOMEM;
    m->cfg = *cfg;
    const int N = m->N = cfg->n_workers, L = m->L = cfg->lag, Z = m->Z = cfg->z_dim, H = m->H = cfg->hidden,
              R = m->R = cfg->rnn_dim;
    const bool bf16 = cfg->mlp_dtype == DKF_DTYPE_BF16;
    const int pad = bf16 ? 64 : 32;  // activation row padding = K granularity of the matrix kernels
    m->Np = round_up(N, pad); m->Zp = round_up(Z, pad); m->Hp = round_up(H, pad); m->Rp = round_up(R, pad);
    const int Smax = cfg->max_samples;
    int rc = DKF_OK;
#define DKF_CHECK(expr) do { rc = (expr); if (rc != DKF_OK) { dkf_free(m); return rc; } } while (0)
#define DKF_CHECK_HIP(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { set_last_hip_error(e_); dkf_free(m); return DKF_EHIP; } } while (0)

    DKF_CHECK(guide_prepare(m->Zp, m->Rp, m->Hp, bf16));

    const float *p = reinterpret_cast<const float *>(static_cast<const char *>(blob) + 32);
    auto take = [&](size_t n) { const float *q = p; p += n; return q; };
    const size_t sN = N, sZ = Z, sH = H, sR = R;
    std::vector<float> bsum(R);
    for (int dir = 0; dir < 2; ++dir) {
        const float *w_ih = take(sR * sN), *b_ih = take(sR), *w_hh = take(sR * sR), *b_hh = take(sR);
        for (int r = 0; r < R; ++r) bsum[r] = b_ih[r] + b_hh[r];
        DKF_CHECK(upload(m, w_ih, sR * sN, dir ? &m->w_ih_b : &m->w_ih_f));
        DKF_CHECK(upload(m, w_hh, sR * sR, dir ? &m->w_hh_b : &m->w_hh_f));
        DKF_CHECK(upload(m, bsum.data(), sR, dir ? &m->bias_b : &m->bias_f));
    }
    RawLayers raw{};
    {
        const float *w, *b;
        w = take(sR * sZ); b = take(sR); DKF_CHECK(pack_layer(m, w, b, R, Z, &m->comb)); raw.comb = w; raw.b_comb = b;
        w = take(sZ * sR); b = take(sZ); DKF_CHECK(pack_layer(m, w, b, Z, R, &m->mu)); raw.mu = w; raw.b_mu = b;
        w = take(sZ * sZ); b = take(sZ); DKF_CHECK(pack_layer(m, w, b, Z, Z, &m->sig)); raw.sig = w; raw.b_sig = b;
        std::vector<float> z0(m->Zp, 0.f);
        std::memcpy(z0.data(), take(sZ), sizeof(float) * sZ);
        DKF_CHECK(upload(m, z0.data(), z0.size(), &m->z0));
        w = take(sH * sZ); b = take(sH); DKF_CHECK(pack_layer(m, w, b, H, Z, &m->gate1)); raw.gate1 = w; raw.b_gate1 = b;
        w = take(sZ * sH); b = take(sZ); DKF_CHECK(pack_layer(m, w, b, Z, H, &m->gate2)); raw.gate2 = w; raw.b_gate2 = b;
        w = take(sH * sZ); b = take(sH); DKF_CHECK(pack_layer(m, w, b, H, Z, &m->prop1)); raw.prop1 = w; raw.b_prop1 = b;
        w = take(sZ * sH); b = take(sZ); DKF_CHECK(pack_layer(m, w, b, Z, H, &m->prop2)); raw.prop2 = w; raw.b_prop2 = b;
        w = take(sZ * sZ); b = take(sZ); DKF_CHECK(pack_layer(m, w, b, Z, Z, &m->lin)); raw.lin = w; raw.b_lin = b;
        w = take(sZ * sZ); b = take(sZ); DKF_CHECK(pack_layer(m, w, b, Z, Z, &m->tscale)); raw.tscale = w; raw.b_tscale = b;
        w = take(sH * sZ); b = take(sH); DKF_CHECK(pack_layer(m, w, b, H, Z, &m->emean1)); raw.emean1 = w; raw.b_emean1 = b;
        w = take(sN * sH); b = take(sN); DKF_CHECK(pack_layer(m, w, b, N, H, &m->emean2)); raw.emean2 = w; raw.b_emean2 = b;
        w = take(sH * sN); b = take(sH); DKF_CHECK(pack_layer(m, w, b, H, N, &m->escale1)); raw.escale1 = w; raw.b_escale1 = b;
        w = take(sN * sH); b = take(sN); DKF_CHECK(pack_layer(m, w, b, N, H, &m->escale2)); raw.escale2 = w; raw.b_escale2 = b;
    }

    m->use_chain = !bf16 && chain_supported(Z, R, H, L, N);
    if (m->use_chain) DKF_CHECK(pack_chain(m, raw));
    m->use_quad = !bf16 && quad_supported(Z, R, H, L, N);
    if (m->use_quad) DKF_CHECK(pack_quad(m, raw));
    // eight wavefronts per workgroup where their exchange buffers fit into LDS next to the window's
    // encodings, else four
    m->split_waves = split_supported(Z, R, H, L, N, 8) ? 8 : 4;
    m->use_split = !bf16 && split_supported(Z, R, H, L, N, m->split_waves);
    if (m->use_split) DKF_CHECK(pack_split(m, raw));
    m->use_gchain = bf16 && gchain_q(Z, R, H) != 0 && m->Zp == 64;
    if (m->use_gchain) DKF_CHECK(pack_gchain(m, raw));
    if (m->use_gchain) DKF_CHECK(pack_emission_frags(m, raw));

    void *q = nullptr;
    DKF_CHECK(dev_alloc(m, m->in_floats() * 4, &q, true)); m->d_in = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)L * R * 4, &q, true)); m->proj_f = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)L * R * 4, &q, true)); m->proj_b = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)L * m->Rp * 4, &q, true)); m->ctx_f = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)L * m->Rp * 4, &q, true)); m->ctx_b = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)Smax * m->Zp * 4, &q, true)); m->z_next = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)Smax * m->Hp * 4, &q, true)); m->hid1 = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)Smax * m->Np * 4, &q, true)); m->mean = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)Smax * m->Hp * 4, &q, true)); m->hid2 = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)Smax * N * 4, &q, true)); m->samples = static_cast<float *>(q);
    m->cutoff_ws_bytes = cutoff_workspace_bytes(Smax, N);
    DKF_CHECK(dev_alloc(m, m->cutoff_ws_bytes, &q, true)); m->cutoff_ws = q;
    DKF_CHECK(dev_alloc(m, 2 * sizeof(int32_t), &q, true)); m->d_cstar = static_cast<int32_t *>(q);
    DKF_CHECK(dev_alloc(m, 4096, &q, true)); m->sink = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, 256, &q, true)); m->fault = static_cast<int32_t *>(q);
    m->xcd_claims = m->fault + 16;
    if (R > 256) DKF_CHECK(filter_xcd_census((R + 63) / 64, &m->same_xcd));  // wide encoders: several workgroups per direction
    DKF_CHECK(dev_alloc(m, (size_t)L * Smax * Z * 4, &q, false)); m->gen_q = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)Smax * Z * 4, &q, false)); m->gen_z = static_cast<float *>(q);
    DKF_CHECK(dev_alloc(m, (size_t)Smax * N * 4, &q, false)); m->gen_x = static_cast<float *>(q);

    for (int i = 0; i < dkf_model::kStagingSlots + 1; ++i) {
        void *h = nullptr;
        DKF_CHECK_HIP(hipHostMalloc(&h, m->in_floats() * 4, hipHostMallocMapped | hipHostMallocCoherent));
        m->host_allocs.push_back(h);
        if (i < dkf_model::kStagingSlots) {
            m->staging[i] = static_cast<float *>(h);
            DKF_CHECK_HIP(hipEventCreateWithFlags(&m->staging_done[i], hipEventDisableTiming));
        } else {
            m->staging_graph = static_cast<float *>(h);
        }
    }
    {
        void *h = nullptr;
        DKF_CHECK_HIP(hipHostMalloc(&h, 4 * sizeof(int32_t), hipHostMallocMapped | hipHostMallocCoherent));
        m->host_allocs.push_back(h);
        m->cstar_host = static_cast<int32_t *>(h);
        std::memset(h, 0, 4 * sizeof(int32_t));
    }
    DKF_CHECK_HIP(hipStreamCreateWithFlags(&m->own_stream, hipStreamNonBlocking));
    m->window.assign((size_t)L * N, 0.f);
    DKF_CHECK_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    DKF_CHECK_HIP(hipDeviceSynchronize());
#undef DKF_CHECK
#undef DKF_CHECK_HIP
    *out = m;
    return DKF_OK;
}

int dkf_reset(dkf_model *m) {
    if (!m) return DKF_EINVAL;
    DKF_HIP_TRY(hipDeviceSynchronize());
    m->pushes = 0;
    m->scale = 0.f;
    std::fill(m->window.begin(), m->window.end(), 0.f);
    return DKF_OK;
}

int dkf_filter_step(dkf_model *m, const float *x_obs, void *stream_) {
    if (!m || !x_obs) return DKF_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int i = m->staging_next;
    if (m->staging_used[i]) DKF_HIP_TRY(hipEventSynchronize(m->staging_done[i]));
    const int status = stage_observation(m, x_obs, 0, m->staging[i]);
    if (status < 0) return status;
    m->staging_next = (i + 1) % dkf_model::kStagingSlots;
    // the first kernel reads the pinned staging slot directly (no copy node) and mirrors it to d_in
    const int rc = launch_filter(filter_args(m, m->staging[i]), true, status == DKF_OK, stream);
    DKF_HIP_TRY(hipEventRecord(m->staging_done[i], stream));
    m->staging_used[i] = true;
    return rc != DKF_OK ? rc : status;
}

int dkf_sample_runtimes(dkf_model *m, int32_t S, const float *eps_q, const float *eps_z, const float *eps_x,
                        uint64_t seed, float *out_samples, const dkf_stage_outputs *stages, void *stream_) {
    if (!m || !out_samples || S < 1 || S > m->cfg.max_samples) return DKF_EINVAL;
    const int n_null = (eps_q == nullptr) + (eps_z == nullptr) + (eps_x == nullptr);
    if (n_null != 0 && n_null != 3) return DKF_EINVAL;
    if (m->pushes < m->L) return DKF_ENOTREADY;
    if (n_null == 3) {
        const int rc = enqueue_noise(m, S, nullptr, seed, static_cast<hipStream_t>(stream_));
        if (rc != DKF_OK) return rc;
        eps_q = m->gen_q; eps_z = m->gen_z; eps_x = m->gen_x;
    }
    return enqueue_sample(m, S, eps_q, eps_z, eps_x, out_samples, stages, static_cast<hipStream_t>(stream_));
}

size_t cutoff_select_workspace(int32_t S, int32_t N) { return cutoff_workspace_bytes(S, N); }

int cutoff_select(const float *samples, int32_t S, int32_t N, int32_t c_min, int32_t c_max, float t_floor,
                  float *out_sorted, int32_t *out_perm, float *out_mean, float *out_omega, int32_t *out_cstar,
                  void *workspace, size_t workspace_bytes, void *stream) {
    return launch_cutoff_select(samples, S, N, c_min, c_max, t_floor, out_sorted, out_perm, out_mean, out_omega,
                                out_cstar, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

int cutoff_select_rate(const float *samples, int32_t S, int32_t N, int32_t c_min, int32_t c_max, float t_floor,
                       float *out_sorted, int32_t *out_perm, float *out_rate, float *out_omega, int32_t *out_cstar,
                       void *workspace, size_t workspace_bytes, void *stream) {
    return launch_cutoff_select(samples, S, N, c_min, c_max, t_floor, out_sorted, out_perm, out_rate, out_omega,
                                out_cstar, workspace, workspace_bytes, static_cast<hipStream_t>(stream), nullptr,
                                nullptr, 1);
}

int cutoff_select_static(const float *samples, int32_t S, int32_t N, int32_t c_min, int32_t c_max, float t_floor,
                         float *out_sorted, int32_t *out_perm, float *out_mean, float *out_omega,
                         int32_t *out_cstar, void *stream) {
    return launch_cutoff_select_static(samples, S, N, c_min, c_max, t_floor, out_sorted, out_perm, out_mean,
                                       out_omega, out_cstar, static_cast<hipStream_t>(stream));
}

size_t cutoff_select_static_max_workspace(void) { return cutoff_static_scratch_bytes(); }

int dkf_decide(dkf_model *m, const float *x_obs, int32_t S, const float *eps_q, const float *eps_z,
               const float *eps_x, uint64_t seed, int32_t *cstar_host, void *stream_) {
    if (!m || !x_obs || !cstar_host || S < 1 || S > m->cfg.max_samples) return DKF_EINVAL;
    const int n_null = (eps_q == nullptr) + (eps_z == nullptr) + (eps_x == nullptr);
    if (n_null != 0 && n_null != 3) return DKF_EINVAL;
    const bool own_noise = n_null == 3;
    hipStream_t stream = stream_ ? static_cast<hipStream_t>(stream_) : m->own_stream;
    // the eager path may still own staging slots on another stream: drain it
    for (int i = 0; i < dkf_model::kStagingSlots; ++i)
        if (m->staging_used[i]) { DKF_HIP_TRY(hipEventSynchronize(m->staging_done[i])); m->staging_used[i] = false; }
    const int status = stage_observation(m, x_obs, seed, m->staging_graph);
    if (status < 0) return status;
    const int32_t ticket = m->ticket = m->ticket == INT32_MAX ? 1 : m->ticket + 1;
    reinterpret_cast<Control *>(m->staging_graph + m->Np)->ticket = ticket;
    if (status == DKF_WARMUP) {
        const int rc = launch_filter(filter_args(m, m->staging_graph), true, false, stream);
        if (rc != DKF_OK) return rc;
        DKF_HIP_TRY(hipStreamSynchronize(stream));
        *cstar_host = m->N;
        return DKF_WARMUP;
    }
    const bool reuse = m->graph_exec && m->graph_S == S && m->graph_eps[0] == eps_q && m->graph_eps[1] == eps_z &&
                       m->graph_eps[2] == eps_x && m->graph_spin_limit == m->spin_limit;
    if (!reuse) {
        drop_graph(m);
        DKF_HIP_TRY(hipStreamSynchronize(stream));
        DKF_HIP_TRY(hipStreamBeginCapture(stream, hipStreamCaptureModeThreadLocal));
        g_capturing++;
        // kernels only: the first one reads the pinned staging buffer, the last one writes the
        // decision into pinned host memory
        int rc = launch_filter(filter_args(m, m->staging_graph), true, true, stream);
        hipError_t e = hipSuccess;
        if (rc == DKF_OK && own_noise) rc = enqueue_noise(m, S, m->ctl_dev(), 0, stream);  // seed travels in the control block
        // where the sampler can, it sorts the rows it has just drawn and hands over their rank sums
        const bool fused_sort = sampler_sorts_rows(m, S);
        float *rank_partial = nullptr;
        uint32_t *rank_done = nullptr;
        if (fused_sort) cutoff_rank_sums_at(m->cutoff_ws, S, m->N, &rank_partial, &rank_done);
        if (rc == DKF_OK)
            rc = own_noise ? enqueue_sample(m, S, m->gen_q, m->gen_z, m->gen_x, m->samples, nullptr, stream, rank_partial, rank_done)
                           : enqueue_sample(m, S, eps_q, eps_z, eps_x, m->samples, nullptr, stream, rank_partial, rank_done);
        if (rc == DKF_OK)
            rc = launch_cutoff_select(m->samples, S, m->N, 1, m->N, 0.f, nullptr, nullptr, nullptr, nullptr,
                                      m->cstar_host, m->cutoff_ws, m->cutoff_ws_bytes, stream, &m->ctl_dev()->ticket,
                                      m->fault, 0, fused_sort ? S / 16 : 0);
        g_capturing--;
        hipGraph_t graph = nullptr;
        e = hipStreamEndCapture(stream, &graph);
        if (rc != DKF_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
        if (e != hipSuccess) { set_last_hip_error(e); return DKF_EHIP; }
        m->graph = graph;
        DKF_HIP_TRY(hipGraphInstantiate(&m->graph_exec, m->graph, nullptr, nullptr, 0));
        m->graph_S = S;
        m->graph_spin_limit = m->spin_limit;
        m->graph_eps[0] = eps_q; m->graph_eps[1] = eps_z; m->graph_eps[2] = eps_x;
    }
    DKF_HIP_TRY(hipGraphLaunch(m->graph_exec, stream));
    m->graph_stream = stream;
    m->graph_launched = true;
    // The last kernel stores this decision's ticket, the status and c* as one 64-bit word into pinned
    // host memory (words 2 and 3 of the box).  Watching for the ticket returns the decision a few
    // microseconds before the runtime's own completion path would; the stream is synchronised as
    // well if the ticket does not show up.
    const uint64_t *word = reinterpret_cast<const uint64_t *>(m->cstar_host + 2);
    uint64_t v = 0;
    bool seen = false;
    for (long spin = 0; spin < kTicketSpins; ++spin) {
        v = __atomic_load_n(word, __ATOMIC_ACQUIRE);
        if ((uint32_t)(v >> 32) == (uint32_t)ticket) { seen = true; break; }
        __builtin_ia32_pause();
    }
    if (!seen) {
        DKF_HIP_TRY(hipStreamSynchronize(stream));
        v = __atomic_load_n(word, __ATOMIC_ACQUIRE);
        if ((uint32_t)(v >> 32) != (uint32_t)ticket) return DKF_EHIP;
    }
    *cstar_host = (int32_t)(v & 0xFFFFu);
    return (int)(int16_t)((v >> 16) & 0xFFFFu);
}

int dkf_decide_trace(dkf_model *m, const float *trace_host, int32_t T, int32_t S, const float *eps_q,
                     const float *eps_z, const float *eps_x, uint64_t seed, int32_t *cstar_host,
                     int32_t *status_host, float *latency_us_host, void *stream_) {
    if (!m || !trace_host || T < 1) return DKF_EINVAL;
    for (int32_t t = 0; t < T; ++t) {
        int32_t c = 0;
        const auto t0 = std::chrono::steady_clock::now();
        const int rc = dkf_decide(m, trace_host + (size_t)t * m->N, S, eps_q, eps_z, eps_x, seed + (uint64_t)t, &c, stream_);
        const auto t1 = std::chrono::steady_clock::now();
        if (rc < 0 && rc != DKF_ESTALLED) return rc;
        if (cstar_host) cstar_host[t] = rc == DKF_ESTALLED ? m->N : c;
        if (status_host) status_host[t] = rc;
        if (latency_us_host) latency_us_host[t] = std::chrono::duration<float, std::micro>(t1 - t0).count();
    }
    return DKF_OK;
}

int dkf_check(dkf_model *m, void *stream_) {
    if (!m) return DKF_EINVAL;
    DKF_HIP_TRY(hipStreamSynchronize(static_cast<hipStream_t>(stream_)));
    int32_t f[3] = {0, 0, 0};
    DKF_HIP_TRY(hipMemcpy(f, m->fault, sizeof f, hipMemcpyDeviceToHost));
    return (f[0] | f[1] | f[2]) != 0 ? DKF_ESTALLED : DKF_OK;
}

int dkf_set_exchange_spin_limit(dkf_model *m, int32_t polls) {
    if (!m || polls < 0) return DKF_EINVAL;
    m->spin_limit = polls;
    return DKF_OK;
}

const float *dkf_decide_samples(const dkf_model *m) { return m ? m->samples : nullptr; }

size_t dkf_impute_workspace(int32_t S, int32_t N) { return impute_workspace_bytes(S, N); }

int dkf_impute_censored(const float *samples, int32_t S, int32_t N, const float *x_obs, const uint8_t *censored,
                        float tau, const float *u, float *x_full, int32_t *n_exceed, void *workspace,
                        size_t workspace_bytes, void *stream) {
    return launch_impute_censored(samples, S, N, x_obs, censored, tau, u, x_full, n_exceed, workspace,
                                  workspace_bytes, static_cast<hipStream_t>(stream));
}

size_t cutoff_rank_spread_workspace(int32_t S, int32_t N) { return rank_spread_workspace_bytes(S, N); }

int cutoff_rank_spread(const float *sorted, int32_t S, int32_t N, const float *mean, float *out_sd, void *workspace,
                       size_t workspace_bytes, void *stream) {
    return launch_rank_spread(sorted, S, N, mean, out_sd, workspace, workspace_bytes,
                              static_cast<hipStream_t>(stream));
}

// state blob: int64 {magic, N, L, pushes}, float scale, float pad, then the ring [L][N]
int dkf_get_state(const dkf_model *m, void *buf, size_t *bytes) {
    if (!m || !bytes) return DKF_EINVAL;
    const size_t need = 4 * sizeof(int64_t) + 2 * sizeof(float) + m->window.size() * sizeof(float);
    if (!buf || *bytes < need) { *bytes = need; return buf ? DKF_EINVAL : DKF_OK; }
    DKF_HIP_TRY(hipDeviceSynchronize());
    char *p = static_cast<char *>(buf);
    const int64_t head[4] = {0x544B4644, m->N, m->L, m->pushes};
    std::memcpy(p, head, sizeof head); p += sizeof head;
    const float sc[2] = {m->scale, 0.f};
    std::memcpy(p, sc, sizeof sc); p += sizeof sc;
    std::memcpy(p, m->window.data(), m->window.size() * sizeof(float));
    *bytes = need;
    return DKF_OK;
}

int dkf_set_state(dkf_model *m, const void *buf, size_t bytes) {
    if (!m || !buf) return DKF_EINVAL;
    const size_t need = 4 * sizeof(int64_t) + 2 * sizeof(float) + m->window.size() * sizeof(float);
    if (bytes != need) return DKF_EINVAL;
    const char *p = static_cast<const char *>(buf);
    int64_t head[4];
    std::memcpy(head, p, sizeof head); p += sizeof head;
    if (head[0] != 0x544B4644 || head[1] != m->N || head[2] != m->L || head[3] < 0) return DKF_EINVAL;
    float sc[2];
    std::memcpy(sc, p, sizeof sc); p += sizeof sc;
    DKF_HIP_TRY(hipDeviceSynchronize());
    std::memcpy(m->window.data(), p, m->window.size() * sizeof(float));
    m->pushes = head[3];
    m->scale = sc[0];
    // rebuild the cached input projections of every stored observation, then the encodings
    const int L = m->L, N = m->N;
    const int stored = m->pushes < L ? (int)m->pushes : L;
    float *dst = m->staging_graph;
    for (int slot = 0; slot < stored; ++slot) {
        std::memcpy(dst, &m->window[(size_t)slot * N], sizeof(float) * N);
        for (int j = N; j < m->Np; ++j) dst[j] = 0.f;
        Control c{};
        c.slot = slot;
        c.count = stored;
        const int newest = (int)((m->pushes + L - 1) % L);
        c.oldest = stored < L ? 0 : (newest + 1) % L;
        c.scale = m->scale;
        c.inv_scale = m->scale > 0.f ? 1.0f / m->scale : 0.f;
        c.seq = next_filter_seq(m);
        std::memcpy(dst + m->Np, &c, sizeof c);
        const int rc = launch_filter(filter_args(m, dst), true, slot == stored - 1 && stored == L, nullptr);
        if (rc != DKF_OK) return rc;
        DKF_HIP_TRY(hipDeviceSynchronize());
    }
    return DKF_OK;
}

int dkf_set_sampler(dkf_model *m, int32_t variant) {
    if (!m || variant < DKF_SAMPLER_AUTO || variant > DKF_SAMPLER_SPLIT) return DKF_EINVAL;
    if (variant == DKF_SAMPLER_SPLIT && !m->use_split) return DKF_EUNSUPPORTED;
    if (variant == DKF_SAMPLER_WAVE16 && !m->use_chain) return DKF_EUNSUPPORTED;
    if (variant == DKF_SAMPLER_WAVE4 && !m->use_quad) return DKF_EUNSUPPORTED;
    if (variant != m->sampler) m->graph_S = 0;  // a captured decision graph holds the old kernels
    m->sampler = variant;
    return DKF_OK;
}

int dkf_sampler_in_use(const dkf_model *m, int32_t S) {
    if (!m || S < 1) return DKF_EINVAL;
    return sampler_for(m, S);
}

int dkf_decide_sorts_in_sampler(const dkf_model *m, int32_t S) {
    if (!m || S < 1) return DKF_EINVAL;
    return sampler_sorts_rows(m, S) ? 1 : 0;
}

int dkf_timing_enable(uint32_t stage_mask) {
    std::lock_guard<std::mutex> lock(g_timing_mu);
    g_timing_mask = stage_mask & ((1u << DKF_NUM_STAGES) - 1);
    return DKF_OK;
}

int dkf_timing_read(int32_t stage, int32_t *launches, double *total_ms) {
    if (stage < 0 || stage >= DKF_NUM_STAGES || !launches || !total_ms) return DKF_EINVAL;
    DKF_HIP_TRY(hipDeviceSynchronize());
    std::lock_guard<std::mutex> lock(g_timing_mu);
    StageRecords &r = g_records[stage];
    double total = 0.0;
    for (int i = 0; i < r.used; ++i) {
        float ms = 0.f;
        DKF_HIP_TRY(hipEventElapsedTime(&ms, r.start[i], r.stop[i]));
        total += ms;
    }
    *launches = r.used;
    *total_ms = total;
    r.used = 0;
    return DKF_OK;
}

}  // extern "C"
