// Sanitizer driver (host only): calls the oracle's and the worker pool's entry points on small
// inputs.  Built with -fsanitize=address,undefined by tests/test_sanitizers_cpu.py together with
// oracle/paac_oracle.cpp and paper_1705_04862_amd/csrc/actors.cpp; any report makes it exit non-zero.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>
#include "../../include/paac_actors.h"

extern "C" {
struct OracleNet { int32_t in_c, in_h, in_w, n_conv, conv_cout[4], conv_k[4], conv_stride[4], fc, n_actions, bf16; };
struct OracleHParams { double gamma, beta, value_coef, lr, rms_alpha, rms_eps, clip_norm; };
struct OracleStats { double policy_loss, entropy, value_loss, total_loss, grad_norm, clip_scale; int32_t nonfinite; };
struct OracleFlipReport { int64_t units[5], flips[5]; double max_abs_pre[5], act_abs_max[5], act_rms[5]; };
uint64_t oracle_param_count(const OracleNet*);
uint64_t oracle_act_per_sample(const OracleNet*);
void oracle_init_params(const OracleNet*, uint64_t, float*);
void oracle_fill_uniforms(uint64_t, uint64_t, float*, uint64_t);
void oracle_select_actions(const OracleNet*, const float*, const uint8_t*, const float*, int, int32_t*, float*, float*, double*);
void oracle_q_select_actions(const OracleNet*, const float*, const uint8_t*, const float*, int, float, int32_t*, double*);
void oracle_forward_f64(const OracleNet*, const double*, const uint8_t*, int, double*, double*, double*);
void oracle_train_step_masked(const OracleNet*, float*, float*, const uint8_t*, const int32_t*, const float*, const uint8_t*,
                              const OracleHParams*, int, int, const uint8_t*, OracleStats*, double*, double*, double*, double*,
                              OracleFlipReport*);
void oracle_q_train_step_masked(const OracleNet*, float*, float*, const uint8_t*, const int32_t*, const float*, const uint8_t*,
                                const OracleHParams*, int, int, const uint8_t*, OracleStats*, double*, double*, double*,
                                OracleFlipReport*);
}

int main() {
    // the small network of the measurement configurations, both storage modes, a ragged little rollout
    for (int bf16 = 0; bf16 < 2; ++bf16) {
        OracleNet net{4, 84, 84, 2, {16, 32, 0, 0}, {8, 4, 0, 0}, {4, 2, 0, 0}, 256, 6, bf16};
        const int T = 2, n_e = 3, B = T * n_e, Bp = (T + 1) * n_e;
        const size_t P = oracle_param_count(&net), APS = oracle_act_per_sample(&net), S = 4 * 84 * 84;
        std::vector<float> params(P), rms(P, 0.01f), u(Bp), rewards(B, 0.f);
        oracle_init_params(&net, 7, params.data());
        oracle_fill_uniforms(11, 3, u.data(), Bp);
        std::vector<uint8_t> states((size_t)Bp * S), dones(B, 0);
        for (size_t i = 0; i < states.size(); ++i) states[i] = (uint8_t)((i * 2654435761u) >> 24);
        dones[1] = 1; rewards[0] = 1.f; rewards[4] = -1.f;
        std::vector<int32_t> actions(B);
        std::vector<float> values(n_e), probs((size_t)n_e * 6);
        std::vector<double> logits((size_t)Bp * 6), vals(Bp), rets(B), grads(P);
        oracle_select_actions(&net, params.data(), states.data(), u.data(), n_e, actions.data(), values.data(), probs.data(), logits.data());
        oracle_q_select_actions(&net, params.data(), states.data(), u.data(), n_e, 0.5f, actions.data() + n_e, logits.data());
        OracleHParams hp{0.99, 0.01, 0.5, 0.0224, 0.99, 0.1, 3.0};
        OracleStats st; OracleFlipReport fr;
        std::vector<double> th(params.begin(), params.end()), acts((size_t)Bp * APS);
        oracle_forward_f64(&net, th.data(), states.data(), Bp, acts.data(), logits.data(), vals.data());
        std::vector<uint8_t> masks(acts.size());
        for (size_t i = 0; i < acts.size(); ++i) masks[i] = acts[i] > 0.0 ? 1 : 0;
        masks[5] ^= 1;
        std::vector<float> p2 = params, r2 = rms;
        oracle_train_step_masked(&net, p2.data(), r2.data(), states.data(), actions.data(), rewards.data(), dones.data(), &hp, T, n_e,
                                 nullptr, &st, grads.data(), logits.data(), vals.data(), rets.data(), nullptr);
        p2 = params; r2 = rms;
        oracle_train_step_masked(&net, p2.data(), r2.data(), states.data(), actions.data(), rewards.data(), dones.data(), &hp, T, n_e,
                                 masks.data(), &st, grads.data(), logits.data(), vals.data(), rets.data(), &fr);
        if (st.nonfinite || fr.flips[0] < 1) { std::printf("unexpected result\n"); return 2; }
        p2 = params; r2 = rms;
        oracle_q_train_step_masked(&net, p2.data(), r2.data(), states.data(), actions.data(), rewards.data(), dones.data(), &hp, T, n_e,
                                   masks.data(), &st, grads.data(), logits.data(), rets.data(), &fr);
    }
    // worker pool: several workers, a negative and an oversized action among the inputs
    paac_actors* a = nullptr;
    if (paac_actors_create(5, 3, 9, 0.3f, 6, &a) != 0) return 3;
    std::vector<uint8_t> obs((size_t)5 * 4 * 84 * 84), dn(5);
    std::vector<float> rw(5);
    std::vector<int32_t> act = {0, -7, 3, 1 << 30, 17};
    paac_actors_reset(a, obs.data());
    for (int i = 0; i < 40; ++i) { act[0] = i; if (paac_actors_step(a, act.data(), obs.data(), rw.data(), dn.data()) != 0) return 4; }
    paac_actors_destroy(a);
    std::printf("sanitizer driver ok\n");
    return 0;
}
