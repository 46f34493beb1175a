// CPU oracle for the PAAC hot path -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// A plain, slow, direct implementation of what one synchronous PAAC iteration computes
// (paper: Section 4 "Parallel Advantage Actor Critic", its two batch-gradient equations,
// and Algorithm 1), written from the definitions: direct nested-loop convolution in NCHW,
// no im2col, no BLAS, no blocking, every sum accumulated in double.  It shares no code,
// header, table or helper with the HIP library; only the tests, the smoke check and the
// benchmark's cpu_baseline leg may load it.
//
// Readings of the paper where it is silent or ambiguous (each also listed in the design notes):
//  * Layer sizes come from the measurement configurations; convolutions use no padding and a
//    ReLU follows every convolution and the hidden fully connected layer (Experiments: one CNN
//    with a softmax policy head and a single linear value node).
//  * rewards[t][e] is the reward for taking actions[t][e] in states[t][e]; the return obeys
//    R_t = r_t + gamma * (1 - done_t) * R_{t+1} with R_{T+1} = V(s_{T+1}) (Algorithm 1, the
//    bootstrap and the backward recursion; the mask generalises its "0 for terminal" rule to a
//    terminal anywhere in the rollout).
//  * The advantage R_t - V(s_t) and the return are constants for differentiation (Section 4:
//    the gradient operator acts on log pi, on H and on V(s_t) only).
//  * The entropy term sits inside the 1/(n_e t_max) mean; the value loss carries a coefficient.
//  * One parameter vector (shared trunk, two heads); one global-L2-norm clip applied before the
//    optimiser; RMSProp is non-centred, has no momentum, starts from zero state and keeps
//    epsilon inside the square root.
//  * ReLU'(0) = 0.  No epsilon inside any logarithm (log-softmax is evaluated stably instead).
//  * The categorical draw is the inverse CDF of the fp32 probabilities accumulated in ascending
//    action order in fp32 (the precision of the kernel that takes the same decision).
//  * ReLU'(pre) = 1[pre > 0] is a binary decision taken by floating point.  A caller may hand in the
//    decisions another implementation took (one byte per unit); the oracle then uses those instead
//    of its own sign test, in the forward pass (unit passes its pre-activation or is zero) and in
//    the backward pass, and reports how many differ from its own and how close to zero its own
//    pre-activation was where they differ.  Nothing else changes.  Without masks every decision is
//    the oracle's own.
//
// Canonical parameter order: for each conv layer W[c_out][c_in][k][k] then b[c_out]; fc W[fc][flat]
// (flat index = c*H*W + y*W + x), fc b; pi W[A][fc], pi b[A]; v W[fc], v b[1].
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#include <algorithm>
#ifdef _OPENMP
#include <omp.h>
#endif

extern "C" {

struct OracleNet {
    int32_t in_c, in_h, in_w;
    int32_t n_conv;
    int32_t conv_cout[4], conv_k[4], conv_stride[4];
    int32_t fc;
    int32_t n_actions;
    int32_t bf16;      // 0: everything in double.  1: emulate bf16 STORAGE of the configurations that
                       // name it: conv/fc weights as used by forward and backward, conv activations and
                       // the gradients handed from layer to layer are rounded to bf16 (round to nearest
                       // even); sums stay in double, master weights and the optimiser stay unrounded.
};

struct OracleHParams {
    double gamma, beta, value_coef, lr, rms_alpha, rms_eps, clip_norm;
};

struct OracleStats {
    double policy_loss, entropy, value_loss, total_loss, grad_norm, clip_scale;
    int32_t nonfinite;
};

// Where supplied ReLU decisions differ from the oracle's own (per layer: conv 1.., then fc).
struct OracleFlipReport {
    int64_t units[5];        // units looked at
    int64_t flips[5];        // units whose supplied decision differs from 1[pre > 0]
    double max_abs_pre[5];   // largest |pre-activation| (the oracle's) among those
    double act_abs_max[5];   // largest |pre-activation| of the layer, for scale
    double act_rms[5];       // root mean square of the layer's pre-activations
};

}  // extern "C"

namespace {

struct Shapes {
    int bf16;
    int n_conv;
    int cin[4], cout[4], k[4], s[4], hin[4], win[4], hout[4], wout[4];
    size_t w_off[4], b_off[4];
    int flat, fc, A;
    size_t fcw_off, fcb_off, piw_off, pib_off, vw_off, vb_off, P;
    size_t act_off[5];   // offsets of each conv output and the fc output inside one sample's record
    size_t act_per_sample;
};

Shapes make_shapes(const OracleNet& n) {
    Shapes s{};
    s.bf16 = n.bf16;
    s.n_conv = n.n_conv;
    int c = n.in_c, h = n.in_h, w = n.in_w;
    size_t off = 0, aoff = 0;
    for (int i = 0; i < n.n_conv; ++i) {
        s.cin[i] = c; s.cout[i] = n.conv_cout[i]; s.k[i] = n.conv_k[i]; s.s[i] = n.conv_stride[i];
        s.hin[i] = h; s.win[i] = w;
        s.hout[i] = (h - s.k[i]) / s.s[i] + 1;
        s.wout[i] = (w - s.k[i]) / s.s[i] + 1;
        s.w_off[i] = off; off += (size_t)s.cout[i] * s.cin[i] * s.k[i] * s.k[i];
        s.b_off[i] = off; off += s.cout[i];
        c = s.cout[i]; h = s.hout[i]; w = s.wout[i];
        s.act_off[i] = aoff; aoff += (size_t)c * h * w;
    }
    s.flat = c * h * w; s.fc = n.fc; s.A = n.n_actions;
    s.act_off[n.n_conv] = aoff; aoff += n.fc;
    s.act_per_sample = aoff;
    s.fcw_off = off; off += (size_t)s.fc * s.flat;
    s.fcb_off = off; off += s.fc;
    s.piw_off = off; off += (size_t)s.A * s.fc;
    s.pib_off = off; off += s.A;
    s.vw_off = off; off += s.fc;
    s.vb_off = off; off += 1;
    s.P = off;
    return s;
}

// Round a value to the nearest bf16 (8-bit significand, ties to even), returned as double.
double round_bf16(double v) {
    float f = (float)v;
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return f;          // inf / nan unchanged
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    std::memcpy(&f, &u, 4);
    return f;
}
inline double q(const Shapes& S, double v) { return S.bf16 ? round_bf16(v) : v; }

// Parameters as the forward and backward passes see them: conv and fc weights rounded to bf16 in the
// bf16 configurations (biases and the two heads stay as they are).
std::vector<double> used_params(const Shapes& S, const double* th) {
    std::vector<double> t(th, th + S.P);
    if (S.bf16) {
        for (int l = 0; l < S.n_conv; ++l)
            for (size_t i = S.w_off[l]; i < S.b_off[l]; ++i) t[i] = round_bf16(t[i]);
        for (size_t i = S.fcw_off; i < S.fcb_off; ++i) t[i] = round_bf16(t[i]);
    }
    return t;
}

// Forward pass of one sample.  x: uint8 [C][H][W].  act: post-ReLU outputs of every conv layer
// and of the fc layer, laid out per Shapes::act_off.  logits[A], *value.
// mask (may be null): one byte per unit of `act`; non-zero = the unit is active.  With a mask the
// unit's output is its pre-activation where the mask says active (whatever its sign) and zero
// elsewhere.  rep (may be null) collects the comparison with the oracle's own sign test.
struct FlipAcc { int64_t units[5], flips[5]; double max_abs_pre[5], abs_max[5], sum_sq[5]; };

inline bool relu_on(const uint8_t* mask, size_t idx, double pre, int layer, FlipAcc* rep) {
    const bool own = pre > 0.0;
    if (!mask) return own;
    const bool given = mask[idx] != 0;
    if (rep) {
        rep->units[layer] += 1;
        const double a = std::fabs(pre);
        if (a > rep->abs_max[layer]) rep->abs_max[layer] = a;
        rep->sum_sq[layer] += pre * pre;
        if (given != own) { rep->flips[layer] += 1; if (a > rep->max_abs_pre[layer]) rep->max_abs_pre[layer] = a; }
    }
    return given;
}

void forward_sample(const Shapes& S, const double* th, const uint8_t* x, double* act,
                    double* logits, double* value, const uint8_t* mask = nullptr, FlipAcc* rep = nullptr) {
    std::vector<double> in0((size_t)S.cin[0] * S.hin[0] * S.win[0]);
    for (size_t i = 0; i < in0.size(); ++i) in0[i] = (double)x[i] / 255.0;
    const double* in = in0.data();
    for (int l = 0; l < S.n_conv; ++l) {
        const double* W = th + S.w_off[l];
        const double* b = th + S.b_off[l];
        double* out = act + S.act_off[l];
        const int K = S.k[l], st = S.s[l], Hi = S.hin[l], Wi = S.win[l];
        for (int co = 0; co < S.cout[l]; ++co)
            for (int oy = 0; oy < S.hout[l]; ++oy)
                for (int ox = 0; ox < S.wout[l]; ++ox) {
                    double acc = b[co];
                    for (int ci = 0; ci < S.cin[l]; ++ci)
                        for (int ky = 0; ky < K; ++ky)
                            for (int kx = 0; kx < K; ++kx)
                                acc += W[(((size_t)co * S.cin[l] + ci) * K + ky) * K + kx] *
                                       in[((size_t)ci * Hi + (oy * st + ky)) * Wi + (ox * st + kx)];
                    const size_t o = ((size_t)co * S.hout[l] + oy) * S.wout[l] + ox;
                    out[o] = relu_on(mask, S.act_off[l] + o, acc, l, rep) ? q(S, acc) : 0.0;
                }
        in = out;
    }
    double* h = act + S.act_off[S.n_conv];
    for (int j = 0; j < S.fc; ++j) {
        double acc = th[S.fcb_off + j];
        for (int i = 0; i < S.flat; ++i) acc += th[S.fcw_off + (size_t)j * S.flat + i] * in[i];
        h[j] = relu_on(mask, S.act_off[S.n_conv] + j, acc, S.n_conv, rep) ? acc : 0.0;
    }
    for (int a = 0; a < S.A; ++a) {
        double acc = th[S.pib_off + a];
        for (int j = 0; j < S.fc; ++j) acc += th[S.piw_off + (size_t)a * S.fc + j] * h[j];
        logits[a] = acc;
    }
    double acc = th[S.vb_off];
    for (int j = 0; j < S.fc; ++j) acc += th[S.vw_off + j] * h[j];
    *value = acc;
}

// Stable softmax: p_k = exp(z_k - max) / sum, log p_k = z_k - max - log(sum).
void softmax(const double* z, int A, double* p, double* logp) {
    double m = z[0];
    for (int k = 1; k < A; ++k) m = std::max(m, z[k]);
    double s = 0.0;
    for (int k = 0; k < A; ++k) s += std::exp(z[k] - m);
    const double ls = std::log(s);
    for (int k = 0; k < A; ++k) {
        if (logp) logp[k] = z[k] - m - ls;
        if (p) p[k] = std::exp(z[k] - m) / s;
    }
}

// Backward pass of one sample: adds this sample's parameter gradient into g (size P).
// dz[A] = dL/dlogits, dv = dL/dV for this sample.
// mask (may be null): the ReLU decisions to use instead of the sign of the stored output.
void backward_sample(const Shapes& S, const double* th, const uint8_t* x, const double* act,
                     const double* dz, double dv, double* g, const uint8_t* mask = nullptr) {
    const double* h = act + S.act_off[S.n_conv];
    std::vector<double> dh(S.fc, 0.0);
    for (int a = 0; a < S.A; ++a) {
        g[S.pib_off + a] += dz[a];
        for (int j = 0; j < S.fc; ++j) {
            g[S.piw_off + (size_t)a * S.fc + j] += dz[a] * h[j];
            dh[j] += dz[a] * th[S.piw_off + (size_t)a * S.fc + j];
        }
    }
    g[S.vb_off] += dv;
    for (int j = 0; j < S.fc; ++j) {
        g[S.vw_off + j] += dv * h[j];
        dh[j] += dv * th[S.vw_off + j];
    }
    // fc layer
    const int L = S.n_conv;
    const double* last = act + S.act_off[L - 1];
    std::vector<double> dcur(S.flat, 0.0);
    for (int j = 0; j < S.fc; ++j) {
        // ReLU'(pre) = 1[pre > 0]; post > 0 iff pre > 0
        if (!(mask ? mask[S.act_off[L] + j] != 0 : h[j] > 0.0)) continue;
        const double d = q(S, dh[j]);
        g[S.fcb_off + j] += d;
        for (int i = 0; i < S.flat; ++i) {
            g[S.fcw_off + (size_t)j * S.flat + i] += d * last[i];
            dcur[i] += d * th[S.fcw_off + (size_t)j * S.flat + i];
        }
    }
    std::vector<double> in0;
    for (int l = L - 1; l >= 0; --l) {
        const double* out = act + S.act_off[l];
        const double* in;
        if (l > 0) in = act + S.act_off[l - 1];
        else {
            in0.resize((size_t)S.cin[0] * S.hin[0] * S.win[0]);
            for (size_t i = 0; i < in0.size(); ++i) in0[i] = (double)x[i] / 255.0;
            in = in0.data();
        }
        const int K = S.k[l], st = S.s[l], Hi = S.hin[l], Wi = S.win[l];
        std::vector<double> din(l > 0 ? (size_t)S.cin[l] * Hi * Wi : 0, 0.0);
        const double* W = th + S.w_off[l];
        for (int co = 0; co < S.cout[l]; ++co)
            for (int oy = 0; oy < S.hout[l]; ++oy)
                for (int ox = 0; ox < S.wout[l]; ++ox) {
                    const size_t o = ((size_t)co * S.hout[l] + oy) * S.wout[l] + ox;
                    if (!(mask ? mask[S.act_off[l] + o] != 0 : out[o] > 0.0)) continue;
                    const double d = q(S, dcur[o]);
                    g[S.b_off[l] + co] += d;
                    for (int ci = 0; ci < S.cin[l]; ++ci)
                        for (int ky = 0; ky < K; ++ky)
                            for (int kx = 0; kx < K; ++kx) {
                                const size_t wi = (((size_t)co * S.cin[l] + ci) * K + ky) * K + kx;
                                const size_t xi = ((size_t)ci * Hi + (oy * st + ky)) * Wi + (ox * st + kx);
                                g[S.w_off[l] + wi] += d * in[xi];
                                if (l > 0) din[xi] += d * W[wi];
                            }
                }
        dcur.swap(din);
    }
}

int n_threads() {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

// Forward over N samples; acts may be null (then activations are discarded per sample).
// masks (may be null): [N][act_per_sample] supplied ReLU decisions; rep (may be null) receives the
// comparison with the oracle's own decisions, summed over the samples.
void forward_batch(const Shapes& S, const double* th_master, const uint8_t* states, int N,
                   double* acts, double* logits, double* values,
                   const uint8_t* masks = nullptr, OracleFlipReport* rep = nullptr) {
    const std::vector<double> used = used_params(S, th_master);
    const double* th = used.data();
    const size_t in_sz = (size_t)S.cin[0] * S.hin[0] * S.win[0];
    FlipAcc total{};
#pragma omp parallel
    {
        std::vector<double> local(acts ? 0 : S.act_per_sample);
        FlipAcc mine{};
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            double* a = acts ? acts + (size_t)n * S.act_per_sample : local.data();
            forward_sample(S, th, states + (size_t)n * in_sz, a, logits + (size_t)n * S.A, values + n,
                           masks ? masks + (size_t)n * S.act_per_sample : nullptr, rep ? &mine : nullptr);
        }
#pragma omp critical
        for (int l = 0; l < 5; ++l) {
            total.units[l] += mine.units[l]; total.flips[l] += mine.flips[l]; total.sum_sq[l] += mine.sum_sq[l];
            total.max_abs_pre[l] = std::max(total.max_abs_pre[l], mine.max_abs_pre[l]);
            total.abs_max[l] = std::max(total.abs_max[l], mine.abs_max[l]);
        }
    }
    if (rep)
        for (int l = 0; l < 5; ++l) {
            rep->units[l] = total.units[l]; rep->flips[l] = total.flips[l];
            rep->max_abs_pre[l] = total.max_abs_pre[l]; rep->act_abs_max[l] = total.abs_max[l];
            rep->act_rms[l] = total.units[l] ? std::sqrt(total.sum_sq[l] / (double)total.units[l]) : 0.0;
        }
}

// Returns (Algorithm 1, bootstrap + backward recursion, with the done mask).
void returns_scan(const float* rewards, const uint8_t* dones, const double* boot, double gamma,
                  int T, int n_e, double* R) {
    for (int e = 0; e < n_e; ++e) {
        double r = boot[e];
        for (int t = T - 1; t >= 0; --t) {
            r = (double)rewards[(size_t)t * n_e + e] + gamma * (dones[(size_t)t * n_e + e] ? 0.0 : 1.0) * r;
            R[(size_t)t * n_e + e] = r;
        }
    }
}

// Losses and their derivatives w.r.t. logits and V for B samples (Section 4, the two batch
// gradients; signs turned into one loss to minimise):
//   L = -(1/B) sum adv * log pi(a) - beta (1/B) sum H + c_v (1/B) sum (R - V)^2,  adv = R - V const.
// dz, dv may be null.  adv_in may be null (then adv = R - V).
void loss_and_grads(const double* logits, const double* values, const double* R, const double* adv_in,
                    const int32_t* actions, int B, int A, double beta, double cv,
                    double* pl, double* ent, double* vl, double* dz, double* dv) {
    double s_pl = 0.0, s_h = 0.0, s_vl = 0.0;
    std::vector<double> p(A), lp(A);
    for (int i = 0; i < B; ++i) {
        softmax(logits + (size_t)i * A, A, p.data(), lp.data());
        double H = 0.0;
        for (int k = 0; k < A; ++k) H -= p[k] * lp[k];
        const double adv = adv_in ? adv_in[i] : R[i] - values[i];
        const int a = actions[i];
        s_pl += -adv * lp[a];
        s_h += H;
        s_vl += (R[i] - values[i]) * (R[i] - values[i]);
        if (dz) {
            for (int k = 0; k < A; ++k) {
                // d(-adv log p_a)/dz_k = -adv (1[k=a] - p_k);  dH/dz_k = -p_k (log p_k + H)
                dz[(size_t)i * A + k] = (-adv * ((k == a ? 1.0 : 0.0) - p[k]) + beta * p[k] * (lp[k] + H)) / B;
            }
        }
        if (dv) dv[i] = 2.0 * cv * (values[i] - R[i]) / B;
    }
    *pl = s_pl / B; *ent = s_h / B; *vl = s_vl / B;
}

// Gradient of the loss over B samples given dz/dv; deterministic reduction over per-thread buffers.
void backward_batch(const Shapes& S, const double* th_master, const uint8_t* states, const double* acts,
                    const double* dz, const double* dv, int B, double* g, const uint8_t* masks = nullptr) {
    const std::vector<double> used = used_params(S, th_master);
    const double* th = used.data();
    const size_t in_sz = (size_t)S.cin[0] * S.hin[0] * S.win[0];
    const int nt = std::max(1, std::min(n_threads(), B));
    std::vector<std::vector<double>> gl(nt, std::vector<double>(S.P, 0.0));
#pragma omp parallel for schedule(static) num_threads(nt)
    for (int tix = 0; tix < nt; ++tix) {
        const int lo = (int)((long long)B * tix / nt), hi = (int)((long long)B * (tix + 1) / nt);
        for (int n = lo; n < hi; ++n)
            backward_sample(S, th, states + (size_t)n * in_sz, acts + (size_t)n * S.act_per_sample,
                            dz + (size_t)n * S.A, dv[n], gl[tix].data(),
                            masks ? masks + (size_t)n * S.act_per_sample : nullptr);
    }
    for (size_t i = 0; i < S.P; ++i) {
        double s = 0.0;
        for (int tix = 0; tix < nt; ++tix) s += gl[tix][i];
        g[i] = s;
    }
}

}  // namespace

extern "C" {

int oracle_threads() { return n_threads(); }
void oracle_set_threads(int n) {
#ifdef _OPENMP
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}

double oracle_round_bf16(double v) { return round_bf16(v); }

uint64_t oracle_param_count(const OracleNet* net) { return make_shapes(*net).P; }
uint64_t oracle_act_per_sample(const OracleNet* net) { return make_shapes(*net).act_per_sample; }

// Forward over N states (uint8 [N][C][H][W]) at double parameters.  acts may be null; otherwise
// [N][act_per_sample] receives every conv output (NCHW, post-ReLU) followed by the fc output.
void oracle_forward_f64(const OracleNet* net, const double* params, const uint8_t* states, int N,
                        double* acts, double* logits, double* values) {
    forward_batch(make_shapes(*net), params, states, N, acts, logits, values);
}

void oracle_softmax_f64(const double* z, int A, double* p, double* logp) { softmax(z, A, p, logp); }

// Inverse-CDF draw in fp32: cdf_k = sum_{j<=k} p_j accumulated in ascending k; the action is the
// smallest k with u < cdf_k, or A-1 if there is none (Algorithm 1: "sample a_t from pi").
int32_t oracle_sample_f32(const float* p, int A, float u) {
    float cdf = 0.0f;
    for (int k = 0; k < A; ++k) {
        cdf = cdf + p[k];
        if (u < cdf) return k;
    }
    return A - 1;
}

void oracle_returns_f64(const float* rewards, const uint8_t* dones, const double* bootstrap,
                        double gamma, int T, int n_e, double* R) {
    returns_scan(rewards, dones, bootstrap, gamma, T, n_e, R);
}

void oracle_loss_f64(const double* logits, const double* values, const double* R, const double* adv,
                     const int32_t* actions, int B, int A, double beta, double cv,
                     double* policy_loss, double* entropy, double* value_loss, double* dz, double* dv) {
    loss_and_grads(logits, values, R, adv, actions, B, A, beta, cv, policy_loss, entropy, value_loss, dz, dv);
}

// The scalar whose gradient the method follows, with the advantage and the return held fixed:
// used by the finite-difference pin.  states: [B] samples.
double oracle_surrogate_loss_f64(const OracleNet* net, const double* params, const uint8_t* states,
                                 const int32_t* actions, const double* adv, const double* R, int B,
                                 double beta, double cv) {
    const Shapes S = make_shapes(*net);
    std::vector<double> logits((size_t)B * S.A), values(B);
    forward_batch(S, params, states, B, nullptr, logits.data(), values.data());
    double pl, ent, vl;
    loss_and_grads(logits.data(), values.data(), R, adv, actions, B, S.A, beta, cv, &pl, &ent, &vl, nullptr, nullptr);
    return pl - beta * ent + cv * vl;
}

// Analytic gradient of the same scalar (advantage and return held fixed) -> grads[P].
void oracle_surrogate_grad_f64(const OracleNet* net, const double* params, const uint8_t* states,
                               const int32_t* actions, const double* adv, const double* R, int B,
                               double beta, double cv, double* grads) {
    const Shapes S = make_shapes(*net);
    std::vector<double> logits((size_t)B * S.A), values(B), acts((size_t)B * S.act_per_sample);
    forward_batch(S, params, states, B, acts.data(), logits.data(), values.data());
    std::vector<double> dz((size_t)B * S.A), dv(B);
    double pl, ent, vl;
    loss_and_grads(logits.data(), values.data(), R, adv, actions, B, S.A, beta, cv, &pl, &ent, &vl, dz.data(), dv.data());
    backward_batch(S, params, states, acts.data(), dz.data(), dv.data(), B, grads);
}

// Backward from given dL/dlogits, dL/dV (for layer-level cross-checks).
void oracle_backward_f64(const OracleNet* net, const double* params, const uint8_t* states, int B,
                         const double* dz, const double* dv, double* grads) {
    const Shapes S = make_shapes(*net);
    std::vector<double> logits((size_t)B * S.A), values(B), acts((size_t)B * S.act_per_sample);
    forward_batch(S, params, states, B, acts.data(), logits.data(), values.data());
    backward_batch(S, params, states, acts.data(), dz, dv, B, grads);
}

// Global-norm clipping: n = ||g||_2 over all parameters, g <- g * min(1, c / n)  (Experiments:
// "gradient clipping"; read as one joint L2 norm).  Returns the scale; *norm_out = n.
double oracle_clip_f64(double* g, uint64_t P, double c, double* norm_out) {
    double ss = 0.0;
    for (uint64_t i = 0; i < P; ++i) ss += g[i] * g[i];
    const double n = std::sqrt(ss);
    double s = 1.0;
    if (n > c) s = c / n;
    if (s != 1.0) for (uint64_t i = 0; i < P; ++i) g[i] *= s;
    if (norm_out) *norm_out = n;
    return s;
}

// RMSProp, epsilon inside the root: g2 <- a g2 + (1-a) g^2 ; theta <- theta - lr g / sqrt(g2 + eps).
void oracle_rmsprop_f64(double* theta, double* g2, const double* g, uint64_t P, double lr,
                        double alpha, double eps) {
    for (uint64_t i = 0; i < P; ++i) {
        g2[i] = alpha * g2[i] + (1.0 - alpha) * g[i] * g[i];
        theta[i] = theta[i] - lr * g[i] / std::sqrt(g2[i] + eps);
    }
}

// paac_select_actions as the oracle computes it: forward over n_e states at fp32-stored
// parameters, softmax in double, probabilities rounded to fp32, inverse-CDF draw in fp32.
void oracle_select_actions(const OracleNet* net, const float* params, const uint8_t* states,
                           const float* uniforms, int n_e, int32_t* actions, float* values,
                           float* probs, double* logits_out) {
    const Shapes S = make_shapes(*net);
    std::vector<double> th(S.P);
    for (size_t i = 0; i < S.P; ++i) th[i] = params[i];
    std::vector<double> logits((size_t)n_e * S.A), v(n_e), p(S.A);
    forward_batch(S, th.data(), states, n_e, nullptr, logits.data(), v.data());
    std::vector<float> pf(S.A);
    for (int e = 0; e < n_e; ++e) {
        softmax(logits.data() + (size_t)e * S.A, S.A, p.data(), nullptr);
        for (int k = 0; k < S.A; ++k) pf[k] = (float)p[k];
        actions[e] = oracle_sample_f32(pf.data(), S.A, uniforms[e]);
        if (values) values[e] = (float)v[e];
        if (probs) for (int k = 0; k < S.A; ++k) probs[(size_t)e * S.A + k] = pf[k];
    }
    if (logits_out) std::memcpy(logits_out, logits.data(), logits.size() * sizeof(double));
}

// paac_train_step as the oracle computes it.  params/rms: fp32 in, updated fp32 out (one rounding
// per step, the storage precision of the method's state).  states uint8 [T+1][n_e][C][H][W];
// actions/rewards/dones [T][n_e] time-major.  Optional double outputs (may be null):
// grads_out[P] = gradient before clipping, logits_out[(T+1) n_e A], values_out[(T+1) n_e],
// returns_out[T n_e].
// masks (may be null): uint8 [(T+1) n_e][act_per_sample], ReLU decisions to use instead of the
// oracle's own (conv outputs in NCHW order followed by the fc units, as in the activation record);
// flips (may be null) reports how they differ from the oracle's own.
void oracle_train_step_masked(const OracleNet* net, float* params, float* rms, const uint8_t* states,
                              const int32_t* actions, const float* rewards, const uint8_t* dones,
                              const OracleHParams* hp, int T, int n_e, const uint8_t* masks,
                              OracleStats* stats, double* grads_out, double* logits_out,
                              double* values_out, double* returns_out, OracleFlipReport* flips);

void oracle_train_step(const OracleNet* net, float* params, float* rms, const uint8_t* states,
                       const int32_t* actions, const float* rewards, const uint8_t* dones,
                       const OracleHParams* hp, int T, int n_e, OracleStats* stats,
                       double* grads_out, double* logits_out, double* values_out, double* returns_out) {
    oracle_train_step_masked(net, params, rms, states, actions, rewards, dones, hp, T, n_e, nullptr, stats,
                             grads_out, logits_out, values_out, returns_out, nullptr);
}

void oracle_train_step_masked(const OracleNet* net, float* params, float* rms, const uint8_t* states,
                              const int32_t* actions, const float* rewards, const uint8_t* dones,
                              const OracleHParams* hp, int T, int n_e, const uint8_t* masks,
                              OracleStats* stats, double* grads_out, double* logits_out,
                              double* values_out, double* returns_out, OracleFlipReport* flips) {
    const Shapes S = make_shapes(*net);
    const int B = T * n_e, Bp = (T + 1) * n_e;
    std::vector<double> th(S.P), g2(S.P);
    for (size_t i = 0; i < S.P; ++i) { th[i] = params[i]; g2[i] = rms[i]; }
    std::vector<double> logits((size_t)Bp * S.A), values(Bp), acts((size_t)Bp * S.act_per_sample);
    forward_batch(S, th.data(), states, Bp, acts.data(), logits.data(), values.data(), masks, flips);
    std::vector<double> R(B);
    returns_scan(rewards, dones, values.data() + B, hp->gamma, T, n_e, R.data());
    std::vector<double> dz((size_t)B * S.A), dv(B), g(S.P);
    double pl, ent, vl;
    loss_and_grads(logits.data(), values.data(), R.data(), nullptr, actions, B, S.A, hp->beta,
                   hp->value_coef, &pl, &ent, &vl, dz.data(), dv.data());
    backward_batch(S, th.data(), states, acts.data(), dz.data(), dv.data(), B, g.data(), masks);
    if (grads_out) std::memcpy(grads_out, g.data(), S.P * sizeof(double));
    double norm = 0.0;
    const double scale = oracle_clip_f64(g.data(), S.P, hp->clip_norm, &norm);
    oracle_rmsprop_f64(th.data(), g2.data(), g.data(), S.P, hp->lr, hp->rms_alpha, hp->rms_eps);
    for (size_t i = 0; i < S.P; ++i) { params[i] = (float)th[i]; rms[i] = (float)g2[i]; }
    if (stats) {
        stats->policy_loss = pl; stats->entropy = ent; stats->value_loss = vl;
        stats->total_loss = pl - hp->beta * ent + hp->value_coef * vl;
        stats->grad_norm = norm; stats->clip_scale = scale;
        stats->nonfinite = (std::isfinite(stats->total_loss) && std::isfinite(norm)) ? 0 : 1;
    }
    if (logits_out) std::memcpy(logits_out, logits.data(), logits.size() * sizeof(double));
    if (values_out) std::memcpy(values_out, values.data(), values.size() * sizeof(double));
    if (returns_out) std::memcpy(returns_out, R.data(), R.size() * sizeof(double));
}

// ------------------------------------------------------------------------------------------------
// Value-based variant of the framework (Section 2.2 "Model-free Value Based Methods": the Bellman
// target r + gamma max_a' Q(s', a') and the squared loss against Q(s, a); Section 3: the framework
// is the same for value-based methods, the policy being implicit in Q).  The network's A head
// outputs are read as Q(s, .); the single value node is not used and receives a zero gradient.
// Readings:
//  * over a rollout of t_max steps the target is the n-step form of the same Bellman backup,
//    R_{T+1} = max_a' Q(s_{T+1}, a'), R_t = r_t + gamma (1 - d_t) R_{t+1}; with t_max = 1 it is the
//    printed one-step target.  The target is a constant for differentiation and uses the same
//    parameters as Q(s, a) (the printed loss has one parameter set theta_i, no target network).
//  * L = c_q (1/B) sum (R - Q(s, a))^2, so dL/dQ(s, a) = -2 c_q (R - Q(s, a)) / B; the factor printed
//    in front of the gradient is a choice of c_q.
//  * behaviour policy: epsilon-greedy on argmax_a Q(s, a) (smallest index among equal maxima) from
//    ONE uniform u per state: u < epsilon explores with action floor((u / epsilon) A), which is
//    uniform given u < epsilon; that quotient is evaluated in fp32, the precision of the kernel
//    that takes the same decision.

// Greedy / explore decision for one state.  q: A action values.
int32_t oracle_q_pick_f32(const double* q, int A, float u, float epsilon) {
    if (u < epsilon) {
        const float x = (u / epsilon) * (float)A;
        int k = (int)x;
        return k < A ? k : A - 1;
    }
    int best = 0;
    for (int k = 1; k < A; ++k) if (q[k] > q[best]) best = k;
    return best;
}

// L = c_q (1/B) sum_i (R_i - Q_i[a_i])^2 ; *msq = (1/B) sum (R - Q)^2 ; dq [B][A] = dL/dQ (may be null).
void oracle_q_loss_f64(const double* Q, const double* R, const int32_t* actions, int B, int A,
                       double cq, double* msq, double* dq) {
    double acc = 0.0;
    for (int i = 0; i < B; ++i) {
        int a = actions[i];
        if (a < 0) a = 0;
        if (a >= A) a = A - 1;
        const double td = R[i] - Q[(size_t)i * A + a];
        acc += td * td;
        if (dq) {
            for (int k = 0; k < A; ++k) dq[(size_t)i * A + k] = 0.0;
            dq[(size_t)i * A + a] = -2.0 * cq * td / (double)B;
        }
    }
    *msq = acc / (double)B;
}

// The scalar whose gradient the variant follows, targets held fixed (finite-difference pin).
double oracle_q_surrogate_loss_f64(const OracleNet* net, const double* params, const uint8_t* states,
                                   const int32_t* actions, const double* R, int B, double cq) {
    const Shapes S = make_shapes(*net);
    std::vector<double> Q((size_t)B * S.A), v(B);
    forward_batch(S, params, states, B, nullptr, Q.data(), v.data());
    double msq;
    oracle_q_loss_f64(Q.data(), R, actions, B, S.A, cq, &msq, nullptr);
    return cq * msq;
}

void oracle_q_surrogate_grad_f64(const OracleNet* net, const double* params, const uint8_t* states,
                                 const int32_t* actions, const double* R, int B, double cq, double* grads) {
    const Shapes S = make_shapes(*net);
    std::vector<double> Q((size_t)B * S.A), v(B), acts((size_t)B * S.act_per_sample);
    forward_batch(S, params, states, B, acts.data(), Q.data(), v.data());
    std::vector<double> dq((size_t)B * S.A), dv(B, 0.0);
    double msq;
    oracle_q_loss_f64(Q.data(), R, actions, B, S.A, cq, &msq, dq.data());
    backward_batch(S, params, states, acts.data(), dq.data(), dv.data(), B, grads);
}

// Action selection of the variant: forward at fp32-stored parameters, epsilon-greedy pick.
// q_out (may be null): [n_e][A] action values in double.
void oracle_q_select_actions(const OracleNet* net, const float* params, const uint8_t* states,
                             const float* uniforms, int n_e, float epsilon, int32_t* actions, double* q_out) {
    const Shapes S = make_shapes(*net);
    std::vector<double> th(S.P);
    for (size_t i = 0; i < S.P; ++i) th[i] = params[i];
    std::vector<double> Q((size_t)n_e * S.A), v(n_e);
    forward_batch(S, th.data(), states, n_e, nullptr, Q.data(), v.data());
    for (int e = 0; e < n_e; ++e) actions[e] = oracle_q_pick_f32(Q.data() + (size_t)e * S.A, S.A, uniforms[e], epsilon);
    if (q_out) std::memcpy(q_out, Q.data(), Q.size() * sizeof(double));
}

// One update of the variant; arguments as oracle_train_step.  stats: value_loss = mean squared TD
// error, total_loss = c_q * value_loss (c_q = hp->value_coef), policy_loss = entropy = 0.
// masks / flips (may be null): supplied ReLU decisions and the report on them, as in
// oracle_train_step_masked.
void oracle_q_train_step_masked(const OracleNet* net, float* params, float* rms, const uint8_t* states,
                                const int32_t* actions, const float* rewards, const uint8_t* dones,
                                const OracleHParams* hp, int T, int n_e, const uint8_t* masks, OracleStats* stats,
                                double* grads_out, double* q_out, double* returns_out, OracleFlipReport* flips);

void oracle_q_train_step(const OracleNet* net, float* params, float* rms, const uint8_t* states,
                         const int32_t* actions, const float* rewards, const uint8_t* dones,
                         const OracleHParams* hp, int T, int n_e, OracleStats* stats,
                         double* grads_out, double* q_out, double* returns_out) {
    oracle_q_train_step_masked(net, params, rms, states, actions, rewards, dones, hp, T, n_e, nullptr, stats,
                               grads_out, q_out, returns_out, nullptr);
}

void oracle_q_train_step_masked(const OracleNet* net, float* params, float* rms, const uint8_t* states,
                                const int32_t* actions, const float* rewards, const uint8_t* dones,
                                const OracleHParams* hp, int T, int n_e, const uint8_t* masks, OracleStats* stats,
                                double* grads_out, double* q_out, double* returns_out, OracleFlipReport* flips) {
    const Shapes S = make_shapes(*net);
    const int B = T * n_e, Bp = (T + 1) * n_e;
    std::vector<double> th(S.P), g2(S.P);
    for (size_t i = 0; i < S.P; ++i) { th[i] = params[i]; g2[i] = rms[i]; }
    std::vector<double> Q((size_t)Bp * S.A), v(Bp), acts((size_t)Bp * S.act_per_sample);
    forward_batch(S, th.data(), states, Bp, acts.data(), Q.data(), v.data(), masks, flips);
    std::vector<double> boot(n_e), R(B);
    for (int e = 0; e < n_e; ++e) {
        const double* q = Q.data() + (size_t)(B + e) * S.A;
        double m = q[0];
        for (int k = 1; k < S.A; ++k) if (q[k] > m) m = q[k];
        boot[e] = m;
    }
    returns_scan(rewards, dones, boot.data(), hp->gamma, T, n_e, R.data());
    std::vector<double> dq((size_t)B * S.A), dv(B, 0.0), g(S.P);
    double msq;
    oracle_q_loss_f64(Q.data(), R.data(), actions, B, S.A, hp->value_coef, &msq, dq.data());
    backward_batch(S, th.data(), states, acts.data(), dq.data(), dv.data(), B, g.data(), masks);
    if (grads_out) std::memcpy(grads_out, g.data(), S.P * sizeof(double));
    double norm = 0.0;
    const double scale = oracle_clip_f64(g.data(), S.P, hp->clip_norm, &norm);
    oracle_rmsprop_f64(th.data(), g2.data(), g.data(), S.P, hp->lr, hp->rms_alpha, hp->rms_eps);
    for (size_t i = 0; i < S.P; ++i) { params[i] = (float)th[i]; rms[i] = (float)g2[i]; }
    if (stats) {
        stats->policy_loss = 0.0; stats->entropy = 0.0; stats->value_loss = msq;
        stats->total_loss = hp->value_coef * msq;
        stats->grad_norm = norm; stats->clip_scale = scale;
        stats->nonfinite = (std::isfinite(stats->total_loss) && std::isfinite(norm)) ? 0 : 1;
    }
    if (q_out) std::memcpy(q_out, Q.data(), Q.size() * sizeof(double));
    if (returns_out) std::memcpy(returns_out, R.data(), R.size() * sizeof(double));
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw 2011, "Parallel random numbers: as easy as 1, 2, 3"):
// counter (c0..c3), key (k0,k1) -> four 32-bit words.
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Uniforms in [0,1) on the 2^-24 grid: element i takes word (i mod 4) of the block whose counter
// is (offset + i/4) as a 64-bit value in (c0,c1), c2 = c3 = 0, key = the 64-bit seed.
void oracle_fill_uniforms(uint64_t seed, uint64_t offset, float* out, uint64_t n) {
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (uint64_t i = 0; i < n; ++i) {
        const uint64_t blk = offset + i / 4;
        const uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u};
        uint32_t w[4];
        oracle_philox4x32_10(ctr, key, w);
        out[i] = (float)(w[i % 4] >> 8) * (1.0f / 16777216.0f);
    }
}

// Glorot-uniform initial parameters from a seed: W ~ U(-l, l), l = sqrt(6 / (fan_in + fan_out)),
// conv fans = channels * k * k; biases zero.  Element i of the canonical vector uses uniform i of
// oracle_fill_uniforms(seed, 0): w = l * (2u - 1) in fp32.
void oracle_init_params(const OracleNet* net, uint64_t seed, float* params) {
    const Shapes S = make_shapes(*net);
    std::vector<float> u(S.P);
    oracle_fill_uniforms(seed, 0, u.data(), S.P);
    auto fill = [&](size_t off, size_t n, double fan_in, double fan_out) {
        const float l = (float)std::sqrt(6.0 / (fan_in + fan_out));
        for (size_t i = 0; i < n; ++i) params[off + i] = l * (2.0f * u[off + i] - 1.0f);
    };
    for (size_t i = 0; i < S.P; ++i) params[i] = 0.0f;
    for (int l = 0; l < S.n_conv; ++l) {
        const double kk = (double)S.k[l] * S.k[l];
        fill(S.w_off[l], (size_t)S.cout[l] * S.cin[l] * S.k[l] * S.k[l], S.cin[l] * kk, S.cout[l] * kk);
    }
    fill(S.fcw_off, (size_t)S.fc * S.flat, S.flat, S.fc);
    fill(S.piw_off, (size_t)S.A * S.fc, S.fc, S.A);
    fill(S.vw_off, (size_t)S.fc, S.fc, 1);
}

}  // extern "C"
