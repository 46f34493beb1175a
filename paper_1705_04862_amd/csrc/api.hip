// C ABI of libpaac: context, workspace carving, parameter layout, the kernel sequences of
// paac_select_actions / paac_train_step, HIP-graph capture and replay, per-kernel timing.
#include "../../include/paac.h"
#include "internal.h"

#include <math.h>
#include <stdio.h>
#include <string.h>
#include <mutex>
#include <string>
#include <vector>

using namespace paac;

namespace paac { thread_local ProfEvents tl_prof = {nullptr, nullptr}; }

// Scratch of paac_select_actions_noalloc: one copy per GPU, held until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress; the address kernels use is looked up once per
// device (scratch_for_device) and passed to them as an argument.
static __device__ __align__(256) unsigned char g_noalloc_scratch[PAAC_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr size_t kAlign = 256;
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of g_noalloc_scratch on `device`, which must be the current device.
hipError_t scratch_for_device(int device, void** out) {
    *out = nullptr;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_noalloc_scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}
constexpr int kHpSlots = 16;
constexpr int kMaxGraphs = 64;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
int pad64(int n) { return (n + 63) / 64 * 64; }

// Internal parameter arena: every tensor starts at a multiple of 64 floats; padding stays zero.
//   conv l : W[k][c_out] with k = (c,ky,kx) for the first layer (uint8 NCHW input) and (ky,kx,c)
//            for later layers (NHWC activations); b[c_out]
//   fc     : W[(y,x,c)][fc], b[fc];  pi: W[A][fc], b[A];  v: W[fc], b[1]
struct Arena {
    int conv_w[3], conv_b[3], fc_w, fc_b, pi_w, pi_b, v_w, v_b;
    int p_int;       // padded length
    size_t P;        // canonical length
    std::vector<int> map;   // canonical index -> arena index
};

Arena make_arena(const NetDesc& n) {
    Arena a{};
    int off = 0;
    auto take = [&](int cnt) { int o = off; off += pad64(cnt); return o; };
    for (int l = 0; l < n.n_conv; ++l) {
        a.conv_w[l] = take(n.conv[l].kk * n.conv[l].cout);
        a.conv_b[l] = take(n.conv[l].cout);
    }
    a.fc_w = take(n.flat * n.fc); a.fc_b = take(n.fc);
    a.pi_w = take(n.n_actions * n.fc); a.pi_b = take(n.n_actions);
    a.v_w = take(n.fc); a.v_b = take(1);
    a.p_int = off;
    for (int l = 0; l < n.n_conv; ++l) {
        const ConvDesc& c = n.conv[l];
        for (int co = 0; co < c.cout; ++co)
            for (int ci = 0; ci < c.cin; ++ci)
                for (int ky = 0; ky < c.ks; ++ky)
                    for (int kx = 0; kx < c.ks; ++kx) {
                        const int k = l == 0 ? (ci * c.ks + ky) * c.ks + kx : (ky * c.ks + kx) * c.cin + ci;
                        a.map.push_back(a.conv_w[l] + k * c.cout + co);
                    }
        for (int co = 0; co < c.cout; ++co) a.map.push_back(a.conv_b[l] + co);
    }
    const ConvDesc& last = n.conv[n.n_conv - 1];
    for (int j = 0; j < n.fc; ++j)
        for (int c = 0; c < last.cout; ++c)
            for (int y = 0; y < last.ho; ++y)
                for (int x = 0; x < last.wo; ++x)
                    a.map.push_back(a.fc_w + ((y * last.wo + x) * last.cout + c) * n.fc + j);
    for (int j = 0; j < n.fc; ++j) a.map.push_back(a.fc_b + j);
    for (int i = 0; i < n.n_actions * n.fc; ++i) a.map.push_back(a.pi_w + i);
    for (int i = 0; i < n.n_actions; ++i) a.map.push_back(a.pi_b + i);
    for (int i = 0; i < n.fc; ++i) a.map.push_back(a.v_w + i);
    a.map.push_back(a.v_b);
    a.P = a.map.size();
    return a;
}

struct Plan {
    int n_e, T, B, Bp;
    Split sel_fc, trn_fc, wg[3], fc_wg;
    int head_chunks, n_loss_blocks;
    bool fused_loss;
};

Plan make_plan(const NetDesc& n, int n_e, int T, bool bf16) {
    Plan p{};
    p.n_e = n_e; p.T = T; p.B = n_e * T; p.Bp = n_e * (T + 1);
    if (bf16) {
        p.sel_fc = plan_split(n.flat, fc_fwd_tiles_bf16(n.arch, n_e), 64, 256);
        p.trn_fc = plan_split(n.flat, fc_fwd_tiles_bf16(n.arch, p.Bp), 64, 256);
        // k-splits of the weight-gradient GEMMs: two workgroups per compute unit for large batches; below 2048
        // transitions half as many, because every split is a partial sum the reduction has to read (n_e = 256:
        // reduction 30.3 -> 25.4 us, fc weight gradient 20.1 -> 22.1 us)
        const int wg_target = p.B < 2048 ? 256 : 512;
        for (int l = 1; l < n.n_conv; ++l) {
            const int direct = conv_wgrad_direct_wgs(n.arch, l, p.B);
            if (direct > 0) { p.wg[l].n = direct; p.wg[l].k_per = 0; }
            else p.wg[l] = plan_split(p.B * n.conv[l].ho * n.conv[l].wo, conv_wgrad_tiles_bf16(n.arch, l), 64, wg_target);
        }
        p.fc_wg = plan_split(p.B, fc_wgrad_tiles_bf16(n.arch), 64, wg_target);
    } else {
        p.sel_fc = plan_split(n.flat, fc_fwd_tiles(n.arch, n_e), 32, fc_fwd_target_wgs(n_e));
        p.trn_fc = plan_split(n.flat, fc_fwd_tiles(n.arch, p.Bp), 32, fc_fwd_target_wgs(p.Bp));
        for (int l = 1; l < n.n_conv; ++l)
            p.wg[l] = plan_split(p.B * n.conv[l].ho * n.conv[l].wo, conv_wgrad_tiles(n.arch, l), 64, 256);
        p.fc_wg = plan_split(p.B, fc_wgrad_tiles(n.arch), 32, 256);
    }
    // the first layer's weight gradient runs in the direct kernel, one partial per workgroup: three
    // (bf16) or one and a half (fp32, larger LDS tile) workgroups per compute unit, at most one per band
    const int c1_cap = bf16 ? 768 : 384;
    p.wg[0].n = 4 * p.B < c1_cap ? 4 * p.B : c1_cap; p.wg[0].k_per = 0;
    p.head_chunks = p.B / 8 < 1 ? 1 : (p.B / 8 > 128 ? 128 : p.B / 8);
    // below 1024 rows the returns + loss work rides in the head-backward launch, which leaves one
    // partial sum of the loss terms per chunk of rows instead of one per block of the loss kernel
    p.fused_loss = heads_bwd_fuses_loss(p.B, n.n_actions, p.T, n.fc);
    p.n_loss_blocks = p.fused_loss ? p.head_chunks : loss_blocks(n_e);
    return p;
}

// Device workspace, carved in one pass (the same pass computes the size).
struct Buffers {
    float *theta, *g2, *grads, *hp, *block_ss, *loss_partials;
    StatsOut* stats;
    void* act[3];           // conv outputs, NHWC, Bp rows (fp32, or bf16 in the bf16 configuration)
    float *fc_partial, *h, *logits, *values, *returns, *dz, *dv;
    void* dh;               // gradient w.r.t. the fc output (same element type as act)
    void* dact[3];          // gradient w.r.t. conv outputs, B rows
    bf16_t *wt[3], *wd[3], *fc_t, *fc_c;   // bf16 weight copies (bf16 configuration only)
    WeightSplits splits;    // fp32 configuration: conv weights as three bf16 parts each
    WeightCopies copies;
    WeightMirrors mirrors;  // what the optimiser keeps up to date: the splits or the copies
    float *pw[3], *pb[3], *fc_pw, *fc_pb, *hd_pw, *hd_pb;
    size_t bytes;
};

Buffers carve(const NetDesc& n, const Arena& a, const Plan& p, bool bf16, char* base) {
    Buffers b{};
    size_t off = 0;
    auto take = [&](size_t floats) {
        float* ptr = base ? reinterpret_cast<float*>(base + off) : nullptr;
        off += align_up(floats * sizeof(float));
        return ptr;
    };
    b.theta = take(a.p_int); b.g2 = take(a.p_int); b.grads = take(a.p_int);
    b.hp = take(HP_COUNT); b.block_ss = take(norm_blocks_cap(a.p_int)); b.loss_partials = take((size_t)p.n_loss_blocks * 4);
    b.stats = reinterpret_cast<StatsOut*>(take(16));
    for (int l = 0; l < n.n_conv; ++l) {
        const size_t per = (size_t)n.conv[l].ho * n.conv[l].wo * n.conv[l].cout;
        b.act[l] = take(bf16 ? (per * p.Bp + 1) / 2 : per * p.Bp);
        b.dact[l] = take(bf16 ? (per * p.B + 1) / 2 : per * p.B);
    }
    const size_t fcp_sel = (size_t)p.sel_fc.n * p.n_e * n.fc, fcp_trn = (size_t)p.trn_fc.n * p.Bp * n.fc;
    b.fc_partial = take(fcp_sel > fcp_trn ? fcp_sel : fcp_trn);
    b.h = take((size_t)p.Bp * n.fc);
    b.logits = take((size_t)p.Bp * n.n_actions); b.values = take(p.Bp); b.returns = take(p.B);
    b.dz = take((size_t)p.B * n.n_actions); b.dv = take(p.B); b.dh = take((size_t)p.B * n.fc);   // sized for fp32
    for (int l = 0; l < n.n_conv; ++l) {
        b.pw[l] = take((size_t)p.wg[l].n * n.conv[l].kk * n.conv[l].cout);
        b.pb[l] = take((size_t)p.wg[l].n * n.conv[l].cout);
    }
    // an unsplit fc weight gradient is written straight into the gradient arena (no partial buffer)
    b.fc_pw = p.fc_wg.n > 1 ? take((size_t)p.fc_wg.n * n.flat * n.fc) : nullptr; b.fc_pb = take((size_t)p.fc_wg.n * n.fc);
    b.hd_pw = take((size_t)p.head_chunks * (n.n_actions + 1) * n.fc);
    b.hd_pb = take((size_t)p.head_chunks * (n.n_actions + 1));
    if (!bf16) {
        WeightSplits& w = b.splits;
        w.n = n.n_conv;
        for (int l = 0; l < n.n_conv; ++l) {
            w.off[l] = a.conv_w[l]; w.K[l] = n.conv[l].kk; w.C[l] = n.conv[l].cout;
            w.dst[l] = reinterpret_cast<bf16_t*>(take(((size_t)3 * w.plane(l) + 1) / 2));
        }
    }
    if (bf16) {
        WeightCopies& w = b.copies;
        auto copy = [&](bf16_t*& dst, int src_off, int K, int C, int cin, int mode) {
            const int count = mode == 3 ? K * 32 : K * C;       // mode 3 pads the columns to 32
            dst = reinterpret_cast<bf16_t*>(take(((size_t)count + 1) / 2));
            w.dst[w.n] = dst; w.start[w.n] = w.total; w.src_off[w.n] = src_off; w.K[w.n] = K; w.C[w.n] = C;
            w.cin[w.n] = cin; w.mode[w.n] = mode; w.total += count; ++w.n;
        };
        for (int l = 0; l < n.n_conv; ++l) {
            copy(b.wt[l], a.conv_w[l], n.conv[l].kk, n.conv[l].cout, n.conv[l].cin, l == 0 ? 3 : 0);
            if (l > 0) copy(b.wd[l], a.conv_w[l], n.conv[l].kk, n.conv[l].cout, n.conv[l].cin, 2);
        }
        copy(b.fc_t, a.fc_w, n.flat, n.fc, 1, 0);
        copy(b.fc_c, a.fc_w, n.flat, n.fc, 1, 1);
    }
    // the optimiser rewrites splits / copies together with theta
    WeightMirrors& m = b.mirrors;
    auto mirror_of = [&](int off_, int K, int C, int cin) -> int {
        for (int i = 0; i < m.n; ++i) if (m.off[i] == off_) return i;
        const int i = m.n++;
        m.off[i] = off_; m.K[i] = K; m.C[i] = C; m.cin[i] = cin;
        return i;
    };
    for (int l = 0; l < b.splits.n; ++l) m.split[mirror_of(b.splits.off[l], b.splits.K[l], b.splits.C[l], n.conv[l].cin)] = b.splits.dst[l];
    for (int q = 0; q < b.copies.n; ++q) {
        const WeightCopies& w = b.copies;
        const int i = mirror_of(w.src_off[q], w.K[q], w.C[q], w.cin[q]);
        const int d = m.copy[i][0] ? 1 : 0;
        m.copy[i][d] = w.dst[q]; m.mode[i][d] = w.mode[q];
    }
    b.bytes = off;
    return b;
}

// The buffers a select call writes besides its outputs (conv outputs of n_e states, fc partial sums),
// carved from `base` the way carve() does; base = nullptr only computes the size.
struct SelectScratch { void* act[3]; float* fc_partial; size_t bytes; };
SelectScratch carve_select_scratch(const NetDesc& n, const Plan& p, bool bf16, char* base) {
    SelectScratch sc{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void* ptr = base ? base + off : nullptr;
        off += align_up(bytes);
        return ptr;
    };
    for (int l = 0; l < n.n_conv; ++l)
        sc.act[l] = take((size_t)n.conv[l].ho * n.conv[l].wo * n.conv[l].cout * p.n_e * (bf16 ? 2 : 4));
    sc.fc_partial = static_cast<float*>(take((size_t)p.sel_fc.n * p.n_e * n.fc * sizeof(float)));
    sc.bytes = off;
    return sc;
}

enum KernelId {
    K_SEL_CONV1, K_SEL_CONV2, K_SEL_CONV3, K_SEL_FC, K_SEL_HEADS,
    K_TRN_CONV1, K_TRN_CONV2, K_TRN_CONV3, K_TRN_FC, K_TRN_HEADS, K_TRN_LOSS, K_TRN_HEADS_BWD,
    K_TRN_FC_WG, K_TRN_FC_DG, K_TRN_CONV3_WG, K_TRN_CONV3_DG, K_TRN_CONV2_WG, K_TRN_CONV2_DG, K_TRN_CONV1_WG,
    K_TRN_GRAD_REDUCE, K_TRN_RMSPROP, K_TRN_BF16W, K_TRN_FC_BWD, K_TRN_CONV3_BWD, K_TRN_CONV2_BWD,
    K_SEL_TRUNK, K_TRN_TRUNK, K_COUNT
};
const char* const kKernelNames[K_COUNT] = {
    "select.conv1_fwd", "select.conv2_fwd", "select.conv3_fwd", "select.fc_fwd", "select.heads_sample",
    "train.conv1_fwd", "train.conv2_fwd", "train.conv3_fwd", "train.fc_fwd", "train.heads_fwd", "train.returns_loss",
    "train.heads_bwd", "train.fc_wgrad", "train.fc_dgrad", "train.conv3_wgrad",
    "train.conv3_dgrad", "train.conv2_wgrad", "train.conv2_dgrad", "train.conv1_wgrad", "train.grad_reduce_norm",
    "train.clip_rmsprop", "train.bf16_weight_copies", "train.fc_bwd", "train.conv3_bwd", "train.conv2_bwd",
    "select.convs_fwd", "train.convs_fwd"};

struct GraphKey {
    int kind;                 // 0 select, 1 train
    const void* p[6];
    int algorithm; float epsilon;
    bool operator==(const GraphKey& o) const {
        return kind == o.kind && algorithm == o.algorithm && epsilon == o.epsilon && memcmp(p, o.p, sizeof(p)) == 0;
    }
};
struct GraphEntry { GraphKey key; hipGraph_t graph; hipGraphExec_t exec; };

}  // namespace

struct paac_ctx {
    paac_config cfg;
    NetDesc net;
    Arena arena;
    Plan plan;
    Buffers buf;
    hipStream_t stream;       // caller's stream: all work is enqueued here
    hipStream_t cap_stream;   // private stream used only for graph capture
    int device;
    void* noalloc_scratch;    // this device's copy of the static scratch array
    bool have_params;
    bool have_train;          // a train step has run since the context was created: its intermediate results exist
    bool cache_on;            // rollout activation cache enabled
    int sel_count;            // select calls since the last train step / parameter load
    int algorithm;            // PAAC_ALG_*
    float epsilon;            // exploration rate of PAAC_ALG_NSTEP_Q
    bool use_graphs, profiling;
    std::vector<GraphEntry> graphs;
    // hyper-parameter staging: pinned ring, one event per slot
    float* hp_pinned;
    hipEvent_t hp_ev[kHpSlots];
    bool hp_ev_used[kHpSlots];
    int hp_next;
    paac_hparams hp_last;
    bool hp_valid;
    // profiling
    struct Pending { int id; hipEvent_t a, b; };
    std::vector<Pending> pending;
    std::vector<hipEvent_t> ev_pool;
    double k_ms[K_COUNT];
    int k_calls[K_COUNT];
    std::string err;
};

namespace {

int fail(paac_ctx* c, int code, const std::string& msg) {
    if (c) c->err = msg;
    return code;
}
#define HIP_TRY(ctx, expr)                                                                              \
    do {                                                                                                \
        hipError_t e__ = (expr);                                                                        \
        if (e__ != hipSuccess)                                                                          \
            return fail(ctx, PAAC_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e__));           \
    } while (0)

int check_config(const paac_config* cfg, std::string* why) {
    if (cfg->arch != PAAC_ARCH_NIPS && cfg->arch != PAAC_ARCH_NATURE) { *why = "arch must be 0 (nips) or 1 (nature)"; return PAAC_E_BADCONFIG; }
    if (cfg->n_e < 1 || cfg->n_e > (1 << 20)) { *why = "n_e out of range"; return PAAC_E_BADCONFIG; }
    if (cfg->t_max < 1 || cfg->t_max > 4096) { *why = "t_max out of range"; return PAAC_E_BADCONFIG; }
    if (cfg->n_actions < 2 || cfg->n_actions > PAAC_MAX_ACTIONS) { *why = "n_actions must be 2..32"; return PAAC_E_BADCONFIG; }
    if (cfg->in_c != 4 || cfg->in_h != 84 || cfg->in_w != 84) { *why = "input must be 4x84x84"; return PAAC_E_BADCONFIG; }
    if (cfg->precision != PAAC_PREC_FP32 && cfg->precision != PAAC_PREC_BF16) { *why = "precision must be 0 (fp32) or 1 (bf16)"; return PAAC_E_BADCONFIG; }
    // row counts are held in int: (t_max+1) n_e 400 output positions must fit
    if ((double)cfg->n_e * (cfg->t_max + 1) * 400.0 * 64.0 > 2.0e9) { *why = "n_e*(t_max+1) too large"; return PAAC_E_BADCONFIG; }
    return PAAC_OK;
}

// ---- profiling helpers ----
hipEvent_t get_event(paac_ctx* c) {
    if (!c->ev_pool.empty()) { hipEvent_t e = c->ev_pool.back(); c->ev_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
int drain_profile(paac_ctx* c) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (auto& p : c->pending) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) { c->k_ms[p.id] += ms; c->k_calls[p.id] += 1; }
        c->ev_pool.push_back(p.a); c->ev_pool.push_back(p.b);
    }
    c->pending.clear();
    return PAAC_OK;
}

struct Launcher {
    paac_ctx* c; hipStream_t s; bool prof; hipError_t err; int err_id;
    template <class F> void run(int id, F&& f) {
        if (err != hipSuccess) return;
        hipEvent_t a = nullptr, b = nullptr;
        if (prof) { a = get_event(c); b = get_event(c); if (a && b) tl_prof = ProfEvents{a, b}; }
        hipError_t e = f();                        // exactly one kernel launch
        tl_prof = ProfEvents{nullptr, nullptr};
        if (prof && a && b) c->pending.push_back({id, a, b});
        if (e != hipSuccess) { err = e; err_id = id; }
    }
};

struct SelectArgs { const uint8_t* states; const float* uniforms; int32_t* actions; float* values; float* probs; };
struct TrainArgs { const uint8_t* states; const int32_t* actions; const float* rewards; const uint8_t* dones; paac_train_stats* stats; };

// fp32 configuration, layers 1..: from this many samples on a launch takes the kernel that works one
// sample per workgroup on exact bf16 parts; below, the tiled fp32 GEMM fills the chip better.
constexpr int kExactMinSamples = 96;

// Forward trunk shared by select and train: convs, fc partial sums.
// `row0`: first row of the activation buffers this launch writes (0, or the slab of a cached rollout).
void enqueue_trunk(paac_ctx* c, const Buffers& b, Launcher& L, const uint8_t* states, int ns, Split fc_split, int id0, int row0) {
    const NetDesc& n = c->net; const Arena& a = c->arena;
    const void* in = states;
    const bool bf16 = c->cfg.precision == PAAC_PREC_BF16;
    auto act_at = [&](int l) {
        const size_t per = (size_t)n.conv[l].ho * n.conv[l].wo * n.conv[l].cout * (bf16 ? 2 : 4);
        return static_cast<char*>(b.act[l]) + (size_t)row0 * per;
    };
    if (!bf16 && ns >= kExactMinSamples && ns <= trunk_fwd_exact_max()) {
        // one workgroup per sample runs all convolutions (exact bf16 parts)
        const bf16_t* w[3] = {}; const float* bs[3] = {}; float* outs[3] = {};
        for (int l = 0; l < n.n_conv; ++l) { w[l] = b.splits.dst[l]; bs[l] = b.theta + a.conv_b[l]; outs[l] = (float*)act_at(l); }
        L.run(id0 == K_SEL_CONV1 ? K_SEL_TRUNK : K_TRN_TRUNK, [&] { return trunk_fwd_exact(L.s, n.arch, states, w, bs, outs, ns); });
        in = outs[n.n_conv - 1];
    } else
    for (int l = 0; l < n.n_conv; ++l) {
        void* out = act_at(l);
        if (bf16) L.run(id0 + l, [&] { return conv_fwd_bf16(L.s, n.arch, l, in, b.wt[l], b.theta + a.conv_b[l], (bf16_t*)out, ns); });
        else if (l == 0)
            L.run(id0, [&] { return conv1_fwd_exact(L.s, n.arch, states, b.splits.dst[0], b.theta + a.conv_b[0], (float*)out, ns); });
        else if (ns >= kExactMinSamples)
            L.run(id0 + l, [&] { return conv_fwd_exact(L.s, n.arch, l, (const float*)in, b.splits.dst[l], b.theta + a.conv_b[l], (float*)out, ns); });
        else L.run(id0 + l, [&] { return conv_fwd(L.s, n.arch, l, in, b.theta + a.conv_w[l], b.theta + a.conv_b[l], (float*)out, ns); });
        in = out;
    }
    if (bf16) L.run(id0 + 3, [&] { return fc_fwd_bf16(L.s, n.arch, (const bf16_t*)in, b.fc_t, b.fc_partial, ns, fc_split); });
    else L.run(id0 + 3, [&] { return fc_fwd(L.s, n.arch, (const float*)in, b.theta + a.fc_w, b.fc_partial, ns, fc_split); });
}

// `slab` >= 0: keep activations, logits and values as rollout slab `slab` of the training buffers.
// `b`: the context's buffers, or a copy whose activation / partial-sum pointers lead elsewhere.
hipError_t enqueue_select(paac_ctx* c, const Buffers& b, hipStream_t s, bool prof, const SelectArgs& x, int slab, int* err_id) {
    Launcher L{c, s, prof, hipSuccess, -1};
    const NetDesc& n = c->net; const Arena& a = c->arena; const Plan& p = c->plan;
    if (prof) delay_us(s, 250);
    const int row0 = slab >= 0 ? slab * p.n_e : 0;
    enqueue_trunk(c, b, L, x.states, p.n_e, p.sel_fc, K_SEL_CONV1, row0);
    HeadsArgs h{};
    h.fc_partial = b.fc_partial; h.n_split = p.sel_fc.n; h.split_stride = (size_t)p.n_e * n.fc;
    h.fc_b = b.theta + a.fc_b; h.pi_w = b.theta + a.pi_w; h.pi_b = b.theta + a.pi_b;
    h.v_w = b.theta + a.v_w; h.v_b = b.theta + a.v_b;
    h.rows = p.n_e; h.A = n.n_actions;
    h.values_out = x.values; h.uniforms = x.uniforms; h.actions_out = x.actions; h.probs_out = x.probs;
    h.algorithm = c->algorithm; h.epsilon = c->epsilon;
    if (slab >= 0) {
        h.h_out = b.h + (size_t)row0 * n.fc; h.logits_out = b.logits + (size_t)row0 * n.n_actions; h.values_copy = b.values + row0;
    }
    L.run(K_SEL_HEADS, [&] { return heads_fwd(L.s, n.fc, h); });
    *err_id = L.err_id;
    return L.err;
}

// `cached`: rows [0, B) of the forward pass were kept by the select calls of this rollout.
hipError_t enqueue_train(paac_ctx* c, hipStream_t s, bool prof, const TrainArgs& x, bool cached, int* err_id) {
    Launcher L{c, s, prof, hipSuccess, -1};
    const NetDesc& n = c->net; const Arena& a = c->arena; const Buffers& b = c->buf; const Plan& p = c->plan;
    const int A = n.n_actions, F = n.fc, last = n.n_conv - 1;
    // forward over all (t_max+1) n_e states: rows [0, B) are the batch, rows [B, Bp) the bootstrap
    if (prof) delay_us(s, 800);
    const int f_row0 = cached ? p.B : 0, f_rows = cached ? p.n_e : p.Bp;      // rows the forward pass still has to compute
    const Split f_split = cached ? p.sel_fc : p.trn_fc;
    const size_t sample_bytes = (size_t)c->cfg.in_c * c->cfg.in_h * c->cfg.in_w;
    enqueue_trunk(c, b, L, x.states + (size_t)f_row0 * sample_bytes, f_rows, f_split, K_TRN_CONV1, f_row0);
    HeadsArgs h{};
    h.fc_partial = b.fc_partial; h.n_split = f_split.n; h.split_stride = (size_t)f_rows * F;
    h.fc_b = b.theta + a.fc_b; h.pi_w = b.theta + a.pi_w; h.pi_b = b.theta + a.pi_b;
    h.v_w = b.theta + a.v_w; h.v_b = b.theta + a.v_b;
    h.rows = f_rows; h.A = A; h.h_out = b.h + (size_t)f_row0 * F; h.logits_out = b.logits + (size_t)f_row0 * A;
    h.values_out = b.values + f_row0;
    L.run(K_TRN_HEADS, [&] { return heads_fwd(L.s, F, h); });
    LossArgs la{};
    la.logits = b.logits; la.values = b.values; la.actions = x.actions; la.rewards = x.rewards; la.dones = x.dones;
    la.hp = b.hp; la.T = p.T; la.n_e = p.n_e; la.A = A;
    la.returns = b.returns; la.dz = b.dz; la.dv = b.dv; la.loss_partials = b.loss_partials;
    la.algorithm = c->algorithm;
    const bool fused_loss = p.fused_loss;
    if (!fused_loss) L.run(K_TRN_LOSS, [&] { return returns_loss(L.s, la); });
    // heads backward
    const bool bf16 = c->cfg.precision == PAAC_PREC_BF16;
    float* const fc_pw = p.fc_wg.n > 1 ? b.fc_pw : b.grads + a.fc_w;
    L.run(K_TRN_HEADS_BWD, [&] {
        return heads_bwd(L.s, F, A, p.B, p.head_chunks, b.dz, b.dv, b.theta + a.pi_w, b.theta + a.v_w, b.h, bf16 ? nullptr : (float*)b.dh,
                         bf16 ? (bf16_t*)b.dh : nullptr, b.hd_pw, b.hd_pb, fused_loss ? &la : nullptr);
    });
    // fc backward
    if (bf16) {
        L.run(K_TRN_FC_WG, [&] { return fc_wgrad_bf16(L.s, n.arch, (const bf16_t*)b.act[last], (const bf16_t*)b.dh, fc_pw, b.fc_pb, p.B, p.fc_wg); });
        L.run(K_TRN_FC_DG, [&] { return fc_dgrad_bf16(L.s, n.arch, (const bf16_t*)b.dh, b.fc_c, (const bf16_t*)b.act[last], (bf16_t*)b.dact[last], p.B); });
    } else {
        L.run(K_TRN_FC_BWD, [&] {
            return fc_bwd(L.s, n.arch, (const float*)b.act[last], (const float*)b.dh, b.theta + a.fc_w, (float*)b.dact[last],
                          fc_pw, b.fc_pb, p.B, p.fc_wg);
        });
    }
    // conv backward, last layer first
    for (int l = last; l >= 0; --l) {
        const void* in = l == 0 ? (const void*)x.states : (const void*)b.act[l - 1];
        const int wg_id = l == 2 ? K_TRN_CONV3_WG : l == 1 ? K_TRN_CONV2_WG : K_TRN_CONV1_WG;
        if (!bf16 && l > 0) {       // fp32: data and weight gradient of the layer share one launch
            L.run(l == 2 ? K_TRN_CONV3_BWD : K_TRN_CONV2_BWD, [&] {
                return conv_bwd(L.s, n.arch, l, (const float*)b.act[l - 1], (const float*)b.dact[l], b.theta + a.conv_w[l],
                                (float*)b.dact[l - 1], b.pw[l], b.pb[l], p.B, p.wg[l]);
            });
            continue;
        }
        if (l == 0)
            L.run(wg_id, [&] { return conv1_wgrad_direct(L.s, n.arch, !bf16, x.states, b.dact[0], b.pw[0], b.pb[0], p.B, p.wg[0].n); });
        else if (bf16) L.run(wg_id, [&] { return conv_wgrad_bf16(L.s, n.arch, l, in, (const bf16_t*)b.dact[l], b.pw[l], b.pb[l], p.B, p.wg[l]); });
        else L.run(wg_id, [&] { return conv_wgrad(L.s, n.arch, l, in, (const float*)b.dact[l], b.pw[l], b.pb[l], p.B, p.wg[l]); });
        if (l > 0) {
            const int dg_id = l == 2 ? K_TRN_CONV3_DG : K_TRN_CONV2_DG;
            if (bf16) L.run(dg_id, [&] { return conv_dgrad_bf16(L.s, n.arch, l, (const bf16_t*)b.dact[l], b.wd[l], (const bf16_t*)b.act[l - 1], (bf16_t*)b.dact[l - 1], p.B); });
            else L.run(dg_id, [&] { return conv_dgrad(L.s, n.arch, l, (const float*)b.dact[l], b.theta + a.conv_w[l], (const float*)b.act[l - 1], (float*)b.dact[l - 1], p.B); });
        }
    }
    // reduce split gradients, global norm, clip + RMSProp
    GradSegments g{};
    auto seg = [&](const float* ptr, int nsplit, size_t stride, int count, int off) {
        g.partial[g.n] = ptr; g.n_split[g.n] = nsplit; g.stride[g.n] = stride; g.count[g.n] = count; g.off[g.n] = off;
        g.padded[g.n] = pad64(count); ++g.n;
    };
    for (int l = 0; l < n.n_conv; ++l) {
        const int wn = n.conv[l].kk * n.conv[l].cout;
        seg(b.pw[l], p.wg[l].n, wn, wn, a.conv_w[l]);
        seg(b.pb[l], p.wg[l].n, n.conv[l].cout, n.conv[l].cout, a.conv_b[l]);
    }
    seg(fc_pw, p.fc_wg.n, (size_t)n.flat * F, n.flat * F, a.fc_w);
    seg(b.fc_pb, p.fc_wg.n, F, F, a.fc_b);
    seg(b.hd_pw, p.head_chunks, (size_t)(A + 1) * F, A * F, a.pi_w);
    seg(b.hd_pb, p.head_chunks, A + 1, A, a.pi_b);
    seg(b.hd_pw + (size_t)A * F, p.head_chunks, (size_t)(A + 1) * F, F, a.v_w);
    seg(b.hd_pb + A, p.head_chunks, A + 1, 1, a.v_b);
    const int n_ss = plan_reduce_blocks(g);
    if (n_ss > norm_blocks_cap(a.p_int)) { *err_id = K_TRN_GRAD_REDUCE; return hipErrorInvalidValue; }
    L.run(K_TRN_GRAD_REDUCE, [&] { return grad_reduce_norm(L.s, g, b.grads, b.block_ss); });
    L.run(K_TRN_RMSPROP, [&] {
        return rmsprop_update(L.s, a.p_int, b.theta, b.g2, b.grads, b.block_ss, n_ss, b.hp, b.loss_partials, p.n_loss_blocks,
                              b.stats, reinterpret_cast<StatsOut*>(x.stats), b.mirrors);
    });
    *err_id = L.err_id;
    return L.err;
}

template <class Enq>
int run_or_replay(paac_ctx* c, const GraphKey& key, Enq&& enq) {
    int err_id = -1;
    if (c->profiling || !c->use_graphs) {
        if (c->profiling && c->pending.size() > 16384) { int r = drain_profile(c); if (r) return r; }
        hipError_t e = enq(c->stream, c->profiling, &err_id);
        if (e != hipSuccess)
            return fail(c, PAAC_E_HIP, std::string("launch of ") + (err_id >= 0 ? kKernelNames[err_id] : "?") + ": " + hipGetErrorString(e));
        return PAAC_OK;
    }
    for (auto& g : c->graphs)
        if (g.key == key) { HIP_TRY(c, hipGraphLaunch(g.exec, c->stream)); return PAAC_OK; }
    if ((int)c->graphs.size() >= kMaxGraphs) {      // too many distinct argument tuples: launch directly
        hipError_t e = enq(c->stream, false, &err_id);
        if (e != hipSuccess) return fail(c, PAAC_E_HIP, std::string("launch: ") + hipGetErrorString(e));
        return PAAC_OK;
    }
    // Capture on the private stream.  It must see everything already enqueued on the caller's stream
    // only at replay time, and the replay is launched on the caller's stream, so no dependency is
    // needed here.
    GraphEntry ge{};
    ge.key = key;
    HIP_TRY(c, hipStreamBeginCapture(c->cap_stream, hipStreamCaptureModeThreadLocal));
    hipError_t e = enq(c->cap_stream, false, &err_id);
    hipError_t e2 = hipStreamEndCapture(c->cap_stream, &ge.graph);
    if (e != hipSuccess || e2 != hipSuccess) {
        if (e2 == hipSuccess && ge.graph) hipGraphDestroy(ge.graph);
        return fail(c, PAAC_E_HIP, std::string("graph capture failed at ") + (err_id >= 0 ? kKernelNames[err_id] : "end") +
                                       ": " + hipGetErrorString(e != hipSuccess ? e : e2));
    }
    hipError_t e3 = hipGraphInstantiate(&ge.exec, ge.graph, nullptr, nullptr, 0);
    if (e3 != hipSuccess) { hipGraphDestroy(ge.graph); return fail(c, PAAC_E_HIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(e3)); }
    c->graphs.push_back(ge);
    HIP_TRY(c, hipGraphLaunch(ge.exec, c->stream));
    return PAAC_OK;
}

int upload_hparams(paac_ctx* c, const paac_hparams* hp) {
    if (c->hp_valid && memcmp(&c->hp_last, hp, sizeof(*hp)) == 0) return PAAC_OK;
    const int slot = c->hp_next;
    c->hp_next = (c->hp_next + 1) % kHpSlots;
    if (c->hp_ev_used[slot]) HIP_TRY(c, hipEventSynchronize(c->hp_ev[slot]));
    float* dst = c->hp_pinned + slot * HP_COUNT;
    dst[HP_GAMMA] = hp->gamma; dst[HP_BETA] = hp->beta; dst[HP_VCOEF] = hp->value_coef; dst[HP_LR] = hp->lr;
    dst[HP_ALPHA] = hp->rms_alpha; dst[HP_EPS] = hp->rms_eps; dst[HP_CLIP] = hp->clip_norm; dst[7] = 0.f;
    HIP_TRY(c, hipMemcpyAsync(c->buf.hp, dst, HP_COUNT * sizeof(float), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipEventRecord(c->hp_ev[slot], c->stream));
    c->hp_ev_used[slot] = true;
    c->hp_last = *hp;
    c->hp_valid = true;
    return PAAC_OK;
}

struct DeviceGuard {
    int prev; bool ok;
    explicit DeviceGuard(int dev) : prev(-1), ok(false) {
        if (hipGetDevice(&prev) == hipSuccess) { ok = (prev == dev) || hipSetDevice(dev) == hipSuccess; }
    }
    ~DeviceGuard() { if (prev >= 0) hipSetDevice(prev); }
};

}  // namespace

extern "C" {

int paac_workspace_bytes(const paac_config* cfg, size_t* bytes_out) {
    if (!cfg || !bytes_out) return PAAC_E_NULL;
    std::string why;
    int r = check_config(cfg, &why);
    if (r) return r;
    const NetDesc n = make_net(cfg->arch, cfg->n_actions);
    const Arena a = make_arena(n);
    const Plan p = make_plan(n, cfg->n_e, cfg->t_max, cfg->precision == PAAC_PREC_BF16);
    *bytes_out = carve(n, a, p, cfg->precision == PAAC_PREC_BF16, nullptr).bytes;
    return PAAC_OK;
}

int paac_create(const paac_config* cfg, void* workspace_dev, size_t workspace_bytes, void* hip_stream, paac_ctx** ctx_out) {
    if (!cfg || !ctx_out) return PAAC_E_NULL;
    *ctx_out = nullptr;
    std::string why;
    int r = check_config(cfg, &why);
    if (r) return r;
    if (!workspace_dev) return PAAC_E_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace_dev) % kAlign != 0) return PAAC_E_WORKSPACE;
    paac_ctx* c = new paac_ctx();
    c->cfg = *cfg;
    c->net = make_net(cfg->arch, cfg->n_actions);
    c->arena = make_arena(c->net);
    c->plan = make_plan(c->net, cfg->n_e, cfg->t_max, cfg->precision == PAAC_PREC_BF16);
    c->buf = carve(c->net, c->arena, c->plan, cfg->precision == PAAC_PREC_BF16, static_cast<char*>(workspace_dev));
    if (c->buf.bytes > workspace_bytes) { delete c; return PAAC_E_WORKSPACE; }
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->have_params = false; c->have_train = false; c->use_graphs = true; c->profiling = false;
    c->algorithm = PAAC_ALG_ACTOR_CRITIC; c->epsilon = 0.f;
    c->hp_next = 0; c->hp_valid = false;
    memset(c->hp_ev_used, 0, sizeof(c->hp_ev_used));
    memset(c->k_ms, 0, sizeof(c->k_ms)); memset(c->k_calls, 0, sizeof(c->k_calls));
    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) e = scratch_for_device(c->device, &c->noalloc_scratch);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->cap_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&c->hp_pinned), kHpSlots * HP_COUNT * sizeof(float), hipHostMallocDefault);
    for (int i = 0; i < kHpSlots && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&c->hp_ev[i], hipEventDisableTiming);
    if (e != hipSuccess) { delete c; return PAAC_E_HIP; }
    *ctx_out = c;
    return PAAC_OK;
}

void paac_destroy(paac_ctx* c) {
    if (!c) return;
    hipStreamSynchronize(c->stream);
    for (auto& g : c->graphs) { hipGraphExecDestroy(g.exec); hipGraphDestroy(g.graph); }
    for (auto& p : c->pending) { hipEventDestroy(p.a); hipEventDestroy(p.b); }
    for (auto e : c->ev_pool) hipEventDestroy(e);
    for (int i = 0; i < kHpSlots; ++i) hipEventDestroy(c->hp_ev[i]);
    if (c->hp_pinned) hipHostFree(c->hp_pinned);
    if (c->cap_stream) hipStreamDestroy(c->cap_stream);
    delete c;
}

size_t paac_param_count(const paac_ctx* c) { return c ? c->arena.P : 0; }

int paac_set_state(paac_ctx* c, const float* params_host, const float* rms_host) {
    if (!c || !params_host) return c ? fail(c, PAAC_E_NULL, "params_host is NULL") : PAAC_E_NULL;
    const Arena& a = c->arena;
    std::vector<float> th(a.p_int, 0.f), g2(a.p_int, 0.f);
    for (size_t i = 0; i < a.P; ++i) {
        th[a.map[i]] = params_host[i];
        if (rms_host) g2[a.map[i]] = rms_host[i];
    }
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(c->buf.theta, th.data(), a.p_int * sizeof(float), hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemcpy(c->buf.g2, g2.data(), a.p_int * sizeof(float), hipMemcpyHostToDevice));
    HIP_TRY(c, hipMemset(c->buf.grads, 0, a.p_int * sizeof(float)));
    if (c->cfg.precision == PAAC_PREC_BF16) HIP_TRY(c, make_bf16_weights(c->stream, c->buf.copies, c->buf.theta));
    else HIP_TRY(c, split_weights(c->stream, c->buf.splits, c->buf.theta));
    HIP_TRY(c, hipDeviceSynchronize());
    c->have_params = true;
    c->sel_count = 0;          // activations cached under the old parameters are stale
    return PAAC_OK;
}

int paac_get_state(paac_ctx* c, float* params_host, float* rms_host, float* grads_host) {
    if (!c) return PAAC_E_NULL;
    if (!c->have_params) return fail(c, PAAC_E_STATE, "no parameters: call paac_init_params or paac_set_state first");
    const Arena& a = c->arena;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    std::vector<float> tmp(a.p_int);
    float* dst[3] = {params_host, rms_host, grads_host};
    const float* src[3] = {c->buf.theta, c->buf.g2, c->buf.grads};
    for (int k = 0; k < 3; ++k) {
        if (!dst[k]) continue;
        HIP_TRY(c, hipMemcpy(tmp.data(), src[k], a.p_int * sizeof(float), hipMemcpyDeviceToHost));
        for (size_t i = 0; i < a.P; ++i) dst[k][i] = tmp[a.map[i]];
    }
    return PAAC_OK;
}

int paac_init_params(paac_ctx* c, uint64_t seed) {
    if (!c) return PAAC_E_NULL;
    const NetDesc& n = c->net;
    const size_t P = c->arena.P;
    std::vector<float> u(P), th(P, 0.f);
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (size_t blk = 0; blk * 4 < P; ++blk) {
        const uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)((uint64_t)blk >> 32), 0u, 0u};
        uint32_t w[4];
        philox4x32_10(ctr, key, w);
        for (int i = 0; i < 4 && blk * 4 + i < P; ++i) u[blk * 4 + i] = (float)(w[i] >> 8) * (1.0f / 16777216.0f);
    }
    size_t off = 0;
    auto glorot = [&](size_t cnt, double fan_in, double fan_out) {
        const float l = (float)sqrt(6.0 / (fan_in + fan_out));
        for (size_t i = 0; i < cnt; ++i) th[off + i] = l * (2.0f * u[off + i] - 1.0f);
        off += cnt;
    };
    for (int l = 0; l < n.n_conv; ++l) {
        const ConvDesc& cv = n.conv[l];
        const double kk = (double)cv.ks * cv.ks;
        glorot((size_t)cv.cout * cv.cin * cv.ks * cv.ks, cv.cin * kk, cv.cout * kk);
        off += cv.cout;
    }
    glorot((size_t)n.fc * n.flat, n.flat, n.fc); off += n.fc;
    glorot((size_t)n.n_actions * n.fc, n.fc, n.n_actions); off += n.n_actions;
    glorot((size_t)n.fc, n.fc, 1); off += 1;
    return paac_set_state(c, th.data(), nullptr);
}

int paac_select_actions(paac_ctx* c, const uint8_t* states_dev, const float* uniforms_dev, int32_t* actions_dev,
                        float* values_dev, float* probs_dev) {
    if (!c) return PAAC_E_NULL;
    if (!states_dev || !uniforms_dev || !actions_dev) return fail(c, PAAC_E_NULL, "states, uniforms and actions are required");
    if (!c->have_params) return fail(c, PAAC_E_STATE, "no parameters: call paac_init_params or paac_set_state first");
    if (reinterpret_cast<uintptr_t>(states_dev) % 4 != 0) return fail(c, PAAC_E_BADCONFIG, "states_dev must be 4-byte aligned");
    DeviceGuard dg(c->device);
    const SelectArgs x{states_dev, uniforms_dev, actions_dev, values_dev, probs_dev};
    // cached rollout: calls 0 .. t_max-1 since the last train step fill slabs 0 .. t_max-1; further calls
    // use the bootstrap slab (the train step recomputes it) and make the cache invalid by their count
    const int slab = c->cache_on ? (c->sel_count < c->plan.T ? c->sel_count : c->plan.T) : -1;
    GraphKey key{};
    key.kind = 0; key.p[0] = states_dev; key.p[1] = uniforms_dev; key.p[2] = actions_dev; key.p[3] = values_dev; key.p[4] = probs_dev;
    key.p[5] = reinterpret_cast<const void*>(static_cast<uintptr_t>(slab + 1));
    key.algorithm = c->algorithm; key.epsilon = c->epsilon;
    const int r = run_or_replay(c, key, [&](hipStream_t s, bool prof, int* id) { return enqueue_select(c, c->buf, s, prof, x, slab, id); });
    if (r == PAAC_OK && c->cache_on && c->sel_count <= c->plan.T) ++c->sel_count;
    return r;
}

int paac_select_actions_noalloc(paac_ctx* c, const uint8_t* states_dev, const float* uniforms_dev, int32_t* actions_dev,
                                float* values_dev, float* probs_dev) {
    if (!c) return PAAC_E_NULL;
    if (!states_dev || !uniforms_dev || !actions_dev) return fail(c, PAAC_E_NULL, "states, uniforms and actions are required");
    if (!c->have_params) return fail(c, PAAC_E_STATE, "no parameters: call paac_init_params or paac_set_state first");
    if (reinterpret_cast<uintptr_t>(states_dev) % 4 != 0) return fail(c, PAAC_E_BADCONFIG, "states_dev must be 4-byte aligned");
    const bool bf16 = c->cfg.precision == PAAC_PREC_BF16;
    const size_t need = carve_select_scratch(c->net, c->plan, bf16, nullptr).bytes;
    if (need > (size_t)PAAC_NOALLOC_SCRATCH_BYTES) {
        char msg[160];
        snprintf(msg, sizeof(msg), "n_e = %d needs %zu bytes of scratch, the static scratch holds %zu: use paac_select_actions",
                 c->cfg.n_e, need, (size_t)PAAC_NOALLOC_SCRATCH_BYTES);
        return fail(c, PAAC_E_WORKSPACE, msg);
    }
    if (!c->noalloc_scratch) return fail(c, PAAC_E_HIP, "static scratch address unknown on this device");
    DeviceGuard dg(c->device);
    const SelectScratch sc = carve_select_scratch(c->net, c->plan, bf16, static_cast<char*>(c->noalloc_scratch));
    Buffers b = c->buf;                      // parameters and their mirrors stay in the workspace
    for (int l = 0; l < c->net.n_conv; ++l) b.act[l] = sc.act[l];
    b.fc_partial = sc.fc_partial;
    const SelectArgs x{states_dev, uniforms_dev, actions_dev, values_dev, probs_dev};
    int err_id = -1;
    const hipError_t e = enqueue_select(c, b, c->stream, false, x, -1, &err_id);
    if (e != hipSuccess)
        return fail(c, PAAC_E_HIP, std::string("launch of ") + (err_id >= 0 ? kKernelNames[err_id] : "?") + ": " + hipGetErrorString(e));
    return PAAC_OK;
}

int paac_train_step(paac_ctx* c, const uint8_t* states_dev, const int32_t* actions_dev, const float* rewards_dev,
                    const uint8_t* dones_dev, const paac_hparams* hp_host, paac_train_stats* stats_dev) {
    if (!c) return PAAC_E_NULL;
    if (!states_dev || !actions_dev || !rewards_dev || !dones_dev || !hp_host)
        return fail(c, PAAC_E_NULL, "states, actions, rewards, dones and hp are required");
    if (!c->have_params) return fail(c, PAAC_E_STATE, "no parameters: call paac_init_params or paac_set_state first");
    if (reinterpret_cast<uintptr_t>(states_dev) % 4 != 0) return fail(c, PAAC_E_BADCONFIG, "states_dev must be 4-byte aligned");
    const paac_hparams& h = *hp_host;
    if (!(h.gamma >= 0.f && h.gamma <= 1.f) || !(h.rms_alpha >= 0.f && h.rms_alpha < 1.f) || !(h.rms_eps > 0.f) ||
        !(h.clip_norm > 0.f) || !isfinite(h.lr) || !isfinite(h.beta) || !isfinite(h.value_coef))
        return fail(c, PAAC_E_BADCONFIG, "hyper-parameter out of range");
    DeviceGuard dg(c->device);
    int r = upload_hparams(c, hp_host);
    if (r) return r;
    const TrainArgs x{states_dev, actions_dev, rewards_dev, dones_dev, stats_dev};
    const bool cached = c->cache_on && c->sel_count == c->plan.T;
    c->sel_count = 0;
    c->have_train = true;
    GraphKey key{};
    key.kind = 1; key.p[0] = states_dev; key.p[1] = actions_dev; key.p[2] = rewards_dev; key.p[3] = dones_dev; key.p[4] = stats_dev;
    key.p[5] = reinterpret_cast<const void*>(static_cast<uintptr_t>(cached ? 1 : 0));
    key.algorithm = c->algorithm; key.epsilon = 0.f;
    return run_or_replay(c, key, [&](hipStream_t s, bool prof, int* id) { return enqueue_train(c, s, prof, x, cached, id); });
}

int paac_get_train_outputs(paac_ctx* c, float* logits_host, float* values_host, float* returns_host) {
    if (!c) return PAAC_E_NULL;
    if (!c->have_train) return fail(c, PAAC_E_STATE, "no train step yet: nothing is stored");
    const Plan& p = c->plan;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (logits_host) HIP_TRY(c, hipMemcpy(logits_host, c->buf.logits, (size_t)p.Bp * c->net.n_actions * sizeof(float), hipMemcpyDeviceToHost));
    if (values_host) HIP_TRY(c, hipMemcpy(values_host, c->buf.values, (size_t)p.Bp * sizeof(float), hipMemcpyDeviceToHost));
    if (returns_host) HIP_TRY(c, hipMemcpy(returns_host, c->buf.returns, (size_t)p.B * sizeof(float), hipMemcpyDeviceToHost));
    return PAAC_OK;
}

int paac_get_train_activations(paac_ctx* c, int layer, int row0, int rows, float* out_host) {
    if (!c) return PAAC_E_NULL;
    if (!out_host) return fail(c, PAAC_E_NULL, "out_host is NULL");
    const NetDesc& n = c->net; const Plan& p = c->plan;
    if (!c->have_train) return fail(c, PAAC_E_STATE, "no train step yet: nothing is stored");
    if (layer < 0 || layer > n.n_conv) return fail(c, PAAC_E_BADCONFIG, "layer out of range");
    if (row0 < 0 || rows < 0 || (long long)row0 + rows > p.Bp) return fail(c, PAAC_E_BADCONFIG, "row range outside the forward batch");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (rows == 0) return PAAC_OK;
    if (layer == n.n_conv) {        // fc output: fp32 in both configurations
        HIP_TRY(c, hipMemcpy(out_host, c->buf.h + (size_t)row0 * n.fc, (size_t)rows * n.fc * sizeof(float), hipMemcpyDeviceToHost));
        return PAAC_OK;
    }
    const bool bf16 = c->cfg.precision == PAAC_PREC_BF16;
    const ConvDesc& cv = n.conv[layer];
    const size_t hw = (size_t)cv.ho * cv.wo, per = hw * cv.cout, esz = bf16 ? 2 : 4;
    const int chunk = 256;          // rows per staging copy
    std::vector<char> tmp((size_t)(rows < chunk ? rows : chunk) * per * esz);
    for (int r = 0; r < rows; r += chunk) {
        const int nr = rows - r < chunk ? rows - r : chunk;
        HIP_TRY(c, hipMemcpy(tmp.data(), static_cast<const char*>(c->buf.act[layer]) + (size_t)(row0 + r) * per * esz,
                             (size_t)nr * per * esz, hipMemcpyDeviceToHost));
        for (int i = 0; i < nr; ++i) {
            float* dst = out_host + (size_t)(r + i) * per;
            for (size_t pos = 0; pos < hw; ++pos)
                for (int ch = 0; ch < cv.cout; ++ch) {
                    const size_t src = ((size_t)i * hw + pos) * cv.cout + ch;    // NHWC on the device
                    float v;
                    if (bf16) {
                        const uint32_t u = (uint32_t)reinterpret_cast<const uint16_t*>(tmp.data())[src] << 16;
                        memcpy(&v, &u, 4);
                    } else v = reinterpret_cast<const float*>(tmp.data())[src];
                    dst[(size_t)ch * hw + pos] = v;                               // NCHW for the caller
                }
        }
    }
    return PAAC_OK;
}

int paac_fill_uniforms(paac_ctx* c, uint64_t seed, uint64_t offset, float* out_dev, size_t n) {
    if (!c) return PAAC_E_NULL;
    if (!out_dev && n) return fail(c, PAAC_E_NULL, "out_dev is NULL");
    DeviceGuard dg(c->device);
    HIP_TRY(c, fill_uniforms(c->stream, seed, offset, out_dev, n));
    return PAAC_OK;
}

int paac_set_activation_cache(paac_ctx* c, int enabled) {
    if (!c) return PAAC_E_NULL;
    c->cache_on = enabled != 0;
    c->sel_count = 0;
    return PAAC_OK;
}

int paac_set_algorithm(paac_ctx* c, int algorithm, float epsilon) {
    if (!c) return PAAC_E_NULL;
    if (algorithm != PAAC_ALG_ACTOR_CRITIC && algorithm != PAAC_ALG_NSTEP_Q) return fail(c, PAAC_E_BADCONFIG, "unknown algorithm");
    if (algorithm == PAAC_ALG_NSTEP_Q && !(epsilon >= 0.f && epsilon <= 1.f)) return fail(c, PAAC_E_BADCONFIG, "epsilon must be in [0, 1]");
    c->algorithm = algorithm;
    c->epsilon = algorithm == PAAC_ALG_NSTEP_Q ? epsilon : 0.f;
    c->sel_count = 0;
    return PAAC_OK;
}

int paac_set_graphs(paac_ctx* c, int use_graphs) {
    if (!c) return PAAC_E_NULL;
    c->use_graphs = use_graphs != 0;
    return PAAC_OK;
}

int paac_set_profiling(paac_ctx* c, int enabled) {
    if (!c) return PAAC_E_NULL;
    int r = drain_profile(c);
    if (r) return r;
    if (enabled && !c->profiling) { memset(c->k_ms, 0, sizeof(c->k_ms)); memset(c->k_calls, 0, sizeof(c->k_calls)); }
    c->profiling = enabled != 0;
    return PAAC_OK;
}

int paac_kernel_times(paac_ctx* c, int cap, const char** name_out, float* ms_out, int32_t* calls_out, int32_t* n_out) {
    if (!c || !name_out || !ms_out || !calls_out || !n_out) return PAAC_E_NULL;
    int r = drain_profile(c);
    if (r) return r;
    int n = 0;
    for (int i = 0; i < K_COUNT && n < cap; ++i) {
        if (c->k_calls[i] == 0) continue;
        name_out[n] = kKernelNames[i]; ms_out[n] = (float)c->k_ms[i]; calls_out[n] = c->k_calls[i]; ++n;
    }
    *n_out = n;
    return PAAC_OK;
}

int paac_flops(const paac_ctx* c, double* select_flops, double* train_flops) {
    if (!c) return PAAC_E_NULL;
    const NetDesc& n = c->net;
    double fwd = 0.0;
    for (int l = 0; l < n.n_conv; ++l) fwd += 2.0 * n.conv[l].ho * n.conv[l].wo * n.conv[l].kk * n.conv[l].cout;
    fwd += 2.0 * n.flat * n.fc + 2.0 * n.fc * (n.n_actions + 1);
    const double conv1 = 2.0 * n.conv[0].ho * n.conv[0].wo * n.conv[0].kk * n.conv[0].cout;
    const double bwd = 2.0 * fwd - conv1;   // weight + data gradient of every layer, no data gradient for the input
    if (select_flops) *select_flops = fwd * c->plan.n_e;
    if (train_flops) *train_flops = fwd * c->plan.Bp + bwd * c->plan.B;
    return PAAC_OK;
}

const char* paac_last_error(const paac_ctx* c) { return c ? c->err.c_str() : "null context"; }

}  // extern "C"
