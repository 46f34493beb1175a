// The non-GEMM kernels of the PAAC step: policy/value heads with softmax and the categorical
// draw (Algorithm 1, action selection), the n-step return scan with advantages, losses and their
// derivatives w.r.t. logits and V (Algorithm 1, bootstrap / recursion / gradient lines; Section 4),
// the head gradients, the split-gradient reduction with the global L2 norm, and the fused
// clip + RMSProp update (Experiments: RMSProp, gradient clipping).  All arithmetic is fp32.
#include "internal.h"
#include <math.h>

namespace paac {

// Wavefront (64-lane) reductions: four DPP steps reduce each row of 16 lanes (quad swaps, half-row
// mirror, row mirror), then the four row results are read with v_readlane and combined.  The result
// is uniform across the wavefront.
template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_mov<0xB1>(v);     // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);     // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);    // row_half_mirror
    v += dpp_mov<0x140>(v);    // row_mirror
    const int i = __float_as_int(v);
    return (__int_as_float(__builtin_amdgcn_readlane(i, 0)) + __int_as_float(__builtin_amdgcn_readlane(i, 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(i, 32)) + __int_as_float(__builtin_amdgcn_readlane(i, 48)));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_mov<0xB1>(v));
    v = fmaxf(v, dpp_mov<0x4E>(v));
    v = fmaxf(v, dpp_mov<0x141>(v));
    v = fmaxf(v, dpp_mov<0x140>(v));
    const int i = __float_as_int(v);
    return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(i, 0)), __int_as_float(__builtin_amdgcn_readlane(i, 16))),
                 fmaxf(__int_as_float(__builtin_amdgcn_readlane(i, 32)), __int_as_float(__builtin_amdgcn_readlane(i, 48))));
}

// ------------------------------------------------------------------------------------ heads
// Action of one state row, taken by a whole wavefront; lane k < A holds head output k, the other
// lanes -inf.  Actor-critic: softmax, then the inverse CDF of the probabilities summed in ascending
// order in fp32.  Value-based variant (Section 2.2: the policy is argmax_a Q(s, a)): epsilon-greedy
// from the one uniform, u < epsilon picks floor(u / epsilon * A), otherwise the smallest index among
// the maxima.
__device__ __forceinline__ void choose_action(const HeadsArgs& a, float z, int lane, int row) {
    const float m = wave_max(z);
    const float u = a.uniforms[row];
    if (a.algorithm == ALG_NSTEP_Q) {
        const unsigned long long eq = __ballot(lane < a.A && z == m);
        int greedy = __ffsll(eq) - 1;
        greedy = greedy < 0 ? 0 : greedy;          // no maximum (NaN outputs): a valid index all the same
        int act = greedy;
        if (u < a.epsilon) {
            const int k = (int)((u / a.epsilon) * (float)a.A);
            act = k < a.A ? k : a.A - 1;
        }
        if (a.probs_out && lane < a.A)
            a.probs_out[(size_t)row * a.A + lane] = a.epsilon / (float)a.A + (lane == greedy ? 1.f - a.epsilon : 0.f);
        if (lane == 0) a.actions_out[row] = act;
        return;
    }
    const float e = lane < a.A ? expf(z - m) : 0.f;
    const float p = e / wave_sum(e);
    if (a.probs_out && lane < a.A) a.probs_out[(size_t)row * a.A + lane] = p;
    float cdf = 0.f;
    int act = a.A - 1;
    bool found = false;
    for (int k = 0; k < a.A; ++k) {            // ascending order, sequential fp32 sum
        cdf = cdf + __int_as_float(__builtin_amdgcn_readlane(__float_as_int(p), k));
        if (!found && u < cdf) { act = k; found = true; }
    }
    if (lane == 0) a.actions_out[row] = act;
}

// One wavefront per state row.  The fc layer's split partial sums are added, bias and ReLU applied,
// then A+1 dot products (policy logits, value) are reduced across the 64 lanes; lane k ends up
// holding logit k.  In select mode the same wavefront computes the softmax and draws the action.
template <int F, int KMAX>                 // KMAX >= A + 1 outputs (logits + the value)
__global__ __launch_bounds__(256) void heads_fwd_kernel(const HeadsArgs a) {
    constexpr int C = F / 256;            // float4 chunks per lane
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = blockIdx.x * 4 + wave;
    if (row >= a.rows) return;
    float4 h[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int col = c * 256 + lane * 4;
        const float* src = a.fc_partial + (size_t)row * F + col;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        int s = 0;
        for (; s + 8 <= a.n_split; s += 8) {          // eight independent loads in flight
            float4 p[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) p[q] = *reinterpret_cast<const float4*>(src + (size_t)(s + q) * a.split_stride);
#pragma unroll
            for (int q = 0; q < 8; ++q) { acc.x += p[q].x; acc.y += p[q].y; acc.z += p[q].z; acc.w += p[q].w; }
        }
        for (; s < a.n_split; ++s) {
            const float4 p = *reinterpret_cast<const float4*>(src + (size_t)s * a.split_stride);
            acc.x += p.x; acc.y += p.y; acc.z += p.z; acc.w += p.w;
        }
        const float4 b = *reinterpret_cast<const float4*>(a.fc_b + col);
        acc.x = fmaxf(acc.x + b.x, 0.f); acc.y = fmaxf(acc.y + b.y, 0.f);
        acc.z = fmaxf(acc.z + b.z, 0.f); acc.w = fmaxf(acc.w + b.w, 0.f);
        h[c] = acc;
        if (a.h_out) *reinterpret_cast<float4*>(a.h_out + (size_t)row * F + col) = acc;
    }
    // all dot products first, then all reductions: the shuffles of different outputs are independent
    // (branch-free: outputs beyond A re-read the value row and are ignored)
    float d[KMAX];
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
        const float* w = k < a.A ? a.pi_w + (size_t)k * F : a.v_w;
        d[k] = 0.f;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const float4 w4 = *reinterpret_cast<const float4*>(w + c * 256 + lane * 4);
            d[k] += h[c].x * w4.x + h[c].y * w4.y + h[c].z * w4.z + h[c].w * w4.w;
        }
    }
    float z = -INFINITY, v = 0.f;
    const float my_b = lane < a.A ? a.pi_b[lane] : 0.f;
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
        const float t = wave_sum(d[k]);
        z = (lane == k && k < a.A) ? t + my_b : z;
        v = (k == a.A) ? t : v;
    }
    v += a.v_b[0];
    if (a.values_out && lane == 0) a.values_out[row] = v;
    if (a.values_copy && lane == 0) a.values_copy[row] = v;
    if (a.logits_out && lane < a.A) a.logits_out[(size_t)row * a.A + lane] = z;
    if (a.uniforms) choose_action(a, z, lane, row);
}

// Up to 2048 rows (every select call of the measurement configurations, the train forward of the
// smaller ones; measured at 1024 rows: 8.3 -> 6.7 us, at 1536: 9.3 -> 8.0 us against one wave per
// row): one workgroup per state row, so that the chain of dependent memory round trips is
// as short as possible.  All loads that do not depend on h (the split partial sums of the row, the
// head weights of this wave's outputs) are issued at once; thread t owns F/256 hidden units, wave w
// the outputs w, w+4, ...; the element-to-lane assignment and the reduction order of a dot product
// are those of heads_fwd_kernel, so both kernels produce the same bits.
template <int F, int KMAX, int SMAX>        // SMAX: splits held in registers at once (loads issued per round, clamped)
__global__ __launch_bounds__(256) void heads_fwd_row_kernel(const HeadsArgs a) {
    constexpr int C = F / 256, U = F / 256, KW = (KMAX + 3) / 4;      // chunks per lane, units per thread, outputs per wave
    __shared__ __attribute__((aligned(16))) float hs[F];
    __shared__ float outs[KMAX + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x;
    // head weights of this wave's outputs (branch-free: outputs beyond A re-read the value row)
    float4 w4[KW][C];
#pragma unroll
    for (int q = 0; q < KW; ++q) {
        const int k = wave + 4 * q;
        const float* w = k < a.A ? a.pi_w + (size_t)k * F : a.v_w;
#pragma unroll
        for (int c = 0; c < C; ++c) w4[q][c] = *reinterpret_cast<const float4*>(w + c * 256 + lane * 4);
    }
    // hidden units tid*U .. tid*U+U-1: split partial sums added in ascending split order
    const float* src = a.fc_partial + (size_t)row * F + tid * U;
    float acc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) acc[u] = 0.f;
    for (int s0 = 0; s0 < a.n_split; s0 += SMAX) {
        float p[SMAX][U];
#pragma unroll
        for (int q = 0; q < SMAX; ++q) {
            const int sidx = min(s0 + q, a.n_split - 1);              // clamped: a valid address, ignored below
            if constexpr (U == 2) {
                const float2 v = *reinterpret_cast<const float2*>(src + (size_t)sidx * a.split_stride);
                p[q][0] = v.x; p[q][1] = v.y;
            } else {
                p[q][0] = src[(size_t)sidx * a.split_stride];
            }
        }
#pragma unroll
        for (int q = 0; q < SMAX; ++q)
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u] += (s0 + q < a.n_split) ? p[q][u] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        acc[u] = fmaxf(acc[u] + a.fc_b[tid * U + u], 0.f);
        hs[tid * U + u] = acc[u];
        if (a.h_out) a.h_out[(size_t)row * F + tid * U + u] = acc[u];
    }
    __syncthreads();
    float4 h[C];
#pragma unroll
    for (int c = 0; c < C; ++c) h[c] = *reinterpret_cast<const float4*>(hs + c * 256 + lane * 4);
#pragma unroll
    for (int q = 0; q < KW; ++q) {
        float d = 0.f;
#pragma unroll
        for (int c = 0; c < C; ++c) d += h[c].x * w4[q][c].x + h[c].y * w4[q][c].y + h[c].z * w4[q][c].z + h[c].w * w4[q][c].w;
        const float t = wave_sum(d);
        const int k = wave + 4 * q;
        if (lane == 0 && k <= a.A && k < KMAX) outs[k] = t;
    }
    __syncthreads();
    if (wave != 0) return;
    const float z = lane < a.A ? outs[lane] + a.pi_b[lane] : -INFINITY;
    const float v = outs[a.A] + a.v_b[0];
    if (a.values_out && lane == 0) a.values_out[row] = v;
    if (a.values_copy && lane == 0) a.values_copy[row] = v;
    if (a.logits_out && lane < a.A) a.logits_out[(size_t)row * a.A + lane] = z;
    if (a.uniforms) choose_action(a, z, lane, row);
}

template <int F, int KMAX> static void launch_heads(hipStream_t s, const HeadsArgs& a) {
    if (a.rows <= 2048) {
        if (a.n_split <= 8) launch_k((heads_fwd_row_kernel<F, KMAX, 8>), dim3(a.rows), dim3(256), s, a);
        else if (a.n_split <= 16) launch_k((heads_fwd_row_kernel<F, KMAX, 16>), dim3(a.rows), dim3(256), s, a);
        else launch_k((heads_fwd_row_kernel<F, KMAX, 32>), dim3(a.rows), dim3(256), s, a);
    }
    else launch_k((heads_fwd_kernel<F, KMAX>), dim3((a.rows + 3) / 4), dim3(256), s, a);
}

hipError_t heads_fwd(hipStream_t s, int F, const HeadsArgs& a) {
    if (a.rows <= 0) return hipErrorInvalidValue;
    const int outs = a.A + 1;
    if (F == 256) {
        if (outs <= 8) launch_heads<256, 8>(s, a);
        else if (outs <= 19) launch_heads<256, 19>(s, a);
        else launch_heads<256, 33>(s, a);
    } else if (F == 512) {
        if (outs <= 8) launch_heads<512, 8>(s, a);
        else if (outs <= 19) launch_heads<512, 19>(s, a);
        else launch_heads<512, 33>(s, a);
    } else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ returns + loss
// A block owns kEnvPerBlock environments.  Phase 1: one thread per environment runs the backward
// recursion R_t = r_t + gamma (1 - d_t) R_{t+1} from R_{T+1} = V(s_{T+1}).  Phase 2: one thread per
// (t, e) row forms adv = R - V, the three loss terms and dL/dlogits, dL/dV.
constexpr int kEnvPerBlock = 32;
int loss_blocks(int n_e) { return (n_e + kEnvPerBlock - 1) / kEnvPerBlock; }

template <int AMAX>
__global__ __launch_bounds__(256) void returns_loss_kernel(const LossArgs a) {
    const int tid = threadIdx.x;
    const int e0 = blockIdx.x * kEnvPerBlock;
    const int ne_blk = min(kEnvPerBlock, a.n_e - e0);
    const int B = a.T * a.n_e;
    const float gamma = a.hp[HP_GAMMA], beta = a.hp[HP_BETA], cv = a.hp[HP_VCOEF];
    if (tid < ne_blk) {
        const int e = e0 + tid;
        float R;
        if (a.algorithm == ALG_NSTEP_Q) {             // Bellman target: R_{T+1} = max_a' Q(s_{T+1}, a')
            const float* q = a.logits + (size_t)(B + e) * a.A;
            R = q[0];
            for (int k = 1; k < a.A; ++k) R = fmaxf(R, q[k]);
        } else {
            R = a.values[B + e];
        }
        for (int t1 = a.T; t1 > 0; t1 -= 8) {          // eight timesteps of loads in flight, then the scan
            float r[8]; uint8_t d[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int t = max(t1 - 1 - q, 0);
                r[q] = a.rewards[t * a.n_e + e]; d[q] = a.dones[t * a.n_e + e];
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int t = t1 - 1 - q;
                if (t >= 0) {
                    R = r[q] + gamma * (d[q] ? 0.f : 1.f) * R;
                    a.returns[t * a.n_e + e] = R;
                }
            }
        }
    }
    __syncthreads();
    float s_pl = 0.f, s_h = 0.f, s_vl = 0.f;
    const float invB = 1.0f / (float)B;
    for (int idx = tid; idx < a.T * ne_blk; idx += 256) {
        const int t = idx / ne_blk, e = e0 + idx % ne_blk;
        const int i = t * a.n_e + e;
        const float* zp = a.logits + (size_t)i * a.A;
        float z[AMAX];
#pragma unroll
        for (int k = 0; k < AMAX; ++k) z[k] = zp[min(k, a.A - 1)];      // clamped: no divergent loads
        const float V = a.values[i], R = a.returns[i], adv = R - V;
        int act = a.actions[i];
        act = act < 0 ? 0 : (act >= a.A ? a.A - 1 : act);
        if (a.algorithm == ALG_NSTEP_Q) {             // L = c (R - Q(s,a))^2 averaged; the value node is unused
            float qa = z[0];
#pragma unroll
            for (int k = 1; k < AMAX; ++k) qa = (k == act) ? z[k] : qa;
            const float td = R - qa;
            s_vl += td * td;
#pragma unroll
            for (int k = 0; k < AMAX; ++k)
                if (k < a.A) a.dz[(size_t)i * a.A + k] = (k == act) ? -2.f * cv * td * invB : 0.f;
            a.dv[i] = 0.f;
            continue;
        }
        float m = z[0];
#pragma unroll
        for (int k = 1; k < AMAX; ++k) m = fmaxf(m, z[k]);
        float ex[AMAX], se = 0.f;
#pragma unroll
        for (int k = 0; k < AMAX; ++k) { ex[k] = k < a.A ? expf(z[k] - m) : 0.f; se += ex[k]; }
        const float lse = logf(se), inv_se = 1.0f / se;
        float H = 0.f, lp_act = 0.f;
#pragma unroll
        for (int k = 0; k < AMAX; ++k) {
            const float lp = z[k] - m - lse;
            H -= (k < a.A) ? ex[k] * inv_se * lp : 0.f;
            lp_act = (k == act) ? lp : lp_act;
        }
        s_pl += -adv * lp_act;
        s_h += H;
        s_vl += (R - V) * (R - V);
#pragma unroll
        for (int k = 0; k < AMAX; ++k) {
            const float lp = z[k] - m - lse, p = ex[k] * inv_se;
            if (k < a.A) a.dz[(size_t)i * a.A + k] = (-adv * ((k == act ? 1.f : 0.f) - p) + beta * p * (lp + H)) * invB;
        }
        a.dv[i] = 2.f * cv * (V - R) * invB;
    }
    // means over the batch: wave sums, then the four waves in order
    __shared__ float red[3][4];
    const float w0 = wave_sum(s_pl * invB), w1 = wave_sum(s_h * invB), w2 = wave_sum(s_vl * invB);
    if ((tid & 63) == 0) { red[0][tid >> 6] = w0; red[1][tid >> 6] = w1; red[2][tid >> 6] = w2; }
    __syncthreads();
    if (tid < 3) a.loss_partials[blockIdx.x * 4 + tid] = (red[tid][0] + red[tid][1]) + (red[tid][2] + red[tid][3]);
}

hipError_t returns_loss(hipStream_t s, const LossArgs& a) {
    const dim3 grid(loss_blocks(a.n_e));
    if (a.A <= 8) launch_k(returns_loss_kernel<8>, grid, dim3(256), s, a);
    else if (a.A <= 18) launch_k(returns_loss_kernel<18>, grid, dim3(256), s, a);
    else launch_k(returns_loss_kernel<32>, grid, dim3(256), s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ returns + loss, one row per wavefront
// The same quantities as returns_loss_kernel for one batch row, computed by a whole wavefront: lane k < A
// works on logit k, the sums over the actions are wave reductions, the return R_t is recomputed from the
// bootstrap value by the recursion over t' = T-1 .. t (lane t' holds r_t' and the terminal flag, T <= 64).
// A row takes a few hundred cycles instead of the few thousand of one thread walking over all actions:
// this is what lets the head-backward launch compute its own coefficients (below).
struct RowIn { float z, V, boot, r; int act; unsigned d; };
struct RowOut { float coef, R, pl, H, vl; };       // coef: dL/dlogit_lane (lane < A), dL/dV (lane A), else 0
// every load of a row (row is uniform in the wavefront and a valid index)
__device__ __forceinline__ RowIn row_load(const LossArgs& a, int row, int lane) {
    const int A = a.A, e = row % a.n_e, B = a.T * a.n_e, lk = min(lane, A - 1), lt = min(lane, a.T - 1);
    RowIn in;
    in.z = a.logits[(size_t)row * A + lk];
    in.V = a.values[row];
    in.act = a.actions[row];
    in.boot = a.algorithm == ALG_NSTEP_Q ? a.logits[(size_t)(B + e) * A + lk] : a.values[B + e];
    in.r = a.rewards[lt * a.n_e + e];
    in.d = a.dones[lt * a.n_e + e];
    return in;
}
__device__ __forceinline__ RowOut row_compute(const LossArgs& a, const RowIn& in, int row, int lane, float gamma, float beta,
                                              float cv, float invB) {
    const int A = a.A, t = row / a.n_e;
    // R_{T+1} = V(s_{T+1}), or max_a' Q(s_{T+1}, a') for the value-based variant
    float R = a.algorithm == ALG_NSTEP_Q ? wave_max(lane < A ? in.boot : -INFINITY) : in.boot;
    for (int tt = a.T - 1; tt >= t; --tt) {
        const float r = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(in.r), tt));
        const unsigned d = (unsigned)__builtin_amdgcn_readlane((int)in.d, tt);
        R = r + gamma * (d ? 0.f : 1.f) * R;
    }
    const int act = in.act < 0 ? 0 : (in.act >= A ? A - 1 : in.act);
    RowOut o;
    o.R = R;
    if (a.algorithm == ALG_NSTEP_Q) {             // L = c (R - Q(s,a))^2 averaged; the value node is unused
        const float td = R - wave_max(lane == act ? in.z : -INFINITY);
        o.coef = lane == act ? -2.f * cv * td * invB : 0.f;
        o.pl = 0.f; o.H = 0.f; o.vl = td * td;
        return o;
    }
    const float m = wave_max(lane < A ? in.z : -INFINITY);
    const float ex = lane < A ? expf(in.z - m) : 0.f;
    const float se = wave_sum(ex);
    const float lp = in.z - m - logf(se), p = ex * (1.0f / se);
    const float H = -wave_sum(lane < A ? p * lp : 0.f);
    const float lp_act = wave_sum(lane == act ? lp : 0.f);          // one non-zero term: exact
    const float adv = R - in.V;
    o.coef = lane < A ? (-adv * ((lane == act ? 1.f : 0.f) - p) + beta * p * (lp + H)) * invB
                      : (lane == A ? 2.f * cv * (in.V - R) * invB : 0.f);
    o.pl = -adv * lp_act; o.H = H; o.vl = adv * adv;
    return o;
}

// ------------------------------------------------------------------------------------ head backward
// Two independent jobs that both start from dz / dv share one launch (at the paper's batch each is a
// few microseconds of latency, and a kernel boundary costs 2.5):
//   blocks [0, n_dh):  dh[row][j] = 1[h > 0] * (sum_a dz[row][a] pi_w[a][j] + dv[row] v_w[j])
//   the others:        partial_w[chunk][a][j] = sum over the chunk's rows of coef(row, a) * h[row][j],
//                      coef = dz (a < A) or dv (a == A); partial_b[chunk][a] = sum of coef.
// dh blocks of both head-backward kernels
__device__ __forceinline__ void heads_dh_block(int F, int A, int rows, const float* dz, const float* dv, const float* pi_w,
                                               const float* v_w, const float* h, float* dh, bf16_t* dh_b) {
    {
        const int F4 = F / 4;
        const int idx = blockIdx.x * 256 + threadIdx.x;
        if (idx >= rows * F4) return;
        const int row = idx / F4, j = (idx % F4) * 4;
        const float4 wv = *reinterpret_cast<const float4*>(v_w + j);
        float4 acc;
        if (F4 % 64 == 0) {
            // a wave works on one row: its A + 1 coefficients are one load (lane k fetches coefficient
            // k) and broadcasts instead of A + 1 loads of the same address by every lane
            const int lane = threadIdx.x & 63, rowu = __builtin_amdgcn_readfirstlane(row);
            const float cv = lane < A ? dz[(size_t)rowu * A + lane] : (lane == A ? dv[rowu] : 0.f);
            const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(cv), A));
            acc = make_float4(d * wv.x, d * wv.y, d * wv.z, d * wv.w);
            for (int k = 0; k < A; ++k) {
                const float g = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(cv), k));
                const float4 w = *reinterpret_cast<const float4*>(pi_w + (size_t)k * F + j);
                acc.x += g * w.x; acc.y += g * w.y; acc.z += g * w.z; acc.w += g * w.w;
            }
        } else {
            const float d = dv[row];
            acc = make_float4(d * wv.x, d * wv.y, d * wv.z, d * wv.w);
            for (int k = 0; k < A; ++k) {
                const float g = dz[(size_t)row * A + k];
                const float4 w = *reinterpret_cast<const float4*>(pi_w + (size_t)k * F + j);
                acc.x += g * w.x; acc.y += g * w.y; acc.z += g * w.z; acc.w += g * w.w;
            }
        }
        const float4 hv = *reinterpret_cast<const float4*>(h + (size_t)row * F + j);
        acc.x = hv.x > 0.f ? acc.x : 0.f; acc.y = hv.y > 0.f ? acc.y : 0.f;
        acc.z = hv.z > 0.f ? acc.z : 0.f; acc.w = hv.w > 0.f ? acc.w : 0.f;
        if (dh_b) {
            auto bf = [](float f) { __bf16 b = (__bf16)f; return (unsigned)__builtin_bit_cast(unsigned short, b); };
            *reinterpret_cast<uint2*>(dh_b + (size_t)row * F + j) = make_uint2(bf(acc.x) | (bf(acc.y) << 16), bf(acc.z) | (bf(acc.w) << 16));
        } else {
            *reinterpret_cast<float4*>(dh + (size_t)row * F + j) = acc;
        }
    }
}

__global__ __launch_bounds__(256) void heads_bwd_kernel(int F, int A, int rows, int n_dh, int rows_per_chunk, const float* dz,
                                                        const float* dv, const float* pi_w, const float* v_w, const float* h,
                                                        float* dh, bf16_t* dh_b, float* pw, float* pb) {
    if ((int)blockIdx.x < n_dh) {
        heads_dh_block(F, A, rows, dz, dv, pi_w, v_w, h, dh, dh_b);
        return;
    }
    // weight-gradient block (x: 256 hidden units, k: output, c: chunk of rows)
    const int wb = blockIdx.x - n_dh, fx = F / 256;
    const int j = (wb % fx) * 256 + threadIdx.x, k = (wb / fx) % (A + 1), c = wb / (fx * (A + 1));
    const int r0 = c * rows_per_chunk, r1 = min(rows, r0 + rows_per_chunk);      // a trailing chunk may be empty: zeros
    float acc = 0.f, accb = 0.f;
    for (int r = r0; r < r1; r += 8) {                 // eight rows of loads in flight
        float g[8], hv[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int rr = min(r + q, r1 - 1);
            g[q] = k < A ? dz[(size_t)rr * A + k] : dv[rr];
            hv[q] = h[(size_t)rr * F + j];
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            if (r + q < r1) { acc += g[q] * hv[q]; accb += g[q]; }
        }
    }
    pw[((size_t)c * (A + 1) + k) * F + j] = acc;
    if (j == 0) pb[c * (A + 1) + k] = accb;
}

// The same for long chunks of rows (large batches).  With one output per block the A + 1 blocks of a
// chunk read the same rows of h again and again (6.7 times the bytes, measured); here a block owns 64
// hidden units of a chunk for all outputs, its four waves take every fourth row, and their sums meet
// in LDS in wave order.
//
// FUSED (batches below 1024 rows, where the returns + loss kernel is one short block and a kernel
// boundary costs as much as its work): no returns + loss launch precedes this one.  Every wavefront
// computes the coefficients of the row it works on itself (row_compute), the first weight-gradient block
// of each chunk of rows also writes what the loss kernel would have written for those rows: returns, dz,
// dv, and the chunk's sums of the three loss terms as loss_partials[chunk].
struct HeadsBwdArgs {
    int F, A, rows, n_dh, rows_per_dh, rows_per_chunk;
    const float* dz; const float* dv; const float* pi_w; const float* v_w; const float* h;
    float* dh; bf16_t* dh_b; float* pw; float* pb;
    LossArgs loss;                                  // FUSED only
};
template <int AMAX, bool FUSED>
__global__ __launch_bounds__(256) void heads_bwd_rows_kernel(const HeadsBwdArgs a) {
    const int F = a.F, A = a.A, rows = a.rows;
    float gamma = 0.f, beta = 0.f, cvc = 0.f, invB = 0.f;
    if constexpr (FUSED) {
        gamma = a.loss.hp[HP_GAMMA]; beta = a.loss.hp[HP_BETA]; cvc = a.loss.hp[HP_VCOEF];
        invB = 1.0f / (float)(a.loss.T * a.loss.n_e);
    }
    if ((int)blockIdx.x < a.n_dh) {
        // dh for rows_per_dh rows: a thread keeps the head weights of its four hidden units in
        // registers for all of them (one row at a time they are fetched again for every row: 20 KB per
        // wave from L2), a wave works on one row at a time, so dz and dv are scalar loads
        const int F4 = F / 4, quad = threadIdx.x % F4, rpi = 256 / F4, j = quad * 4;
        const int sub = __builtin_amdgcn_readfirstlane(threadIdx.x / F4);      // F4 is a multiple of 64: uniform in a wave
        const int lane = threadIdx.x & 63;
        const int row_end = min(rows, ((int)blockIdx.x + 1) * a.rows_per_dh);
        const int row_first = blockIdx.x * a.rows_per_dh + sub;
        RowIn in0{};
        if constexpr (FUSED) in0 = row_load(a.loss, min(row_first, rows - 1), lane);      // the first row's inputs go out with the weights
        float4 w[AMAX];
#pragma unroll
        for (int k = 0; k < AMAX; ++k) w[k] = *reinterpret_cast<const float4*>(a.pi_w + (size_t)min(k, A - 1) * F + j);
        const float4 wv = *reinterpret_cast<const float4*>(a.v_w + j);
#pragma unroll 4
        for (int row = row_first; row < row_end; row += rpi) {
            const float4 hv = *reinterpret_cast<const float4*>(a.h + (size_t)row * F + j);
            // the row's A + 1 coefficients: one load (lane k fetches coefficient k), then broadcasts
            float cv;
            if constexpr (FUSED) {
                const RowIn in = row == row_first ? in0 : row_load(a.loss, row, lane);
                cv = row_compute(a.loss, in, row, lane, gamma, beta, cvc, invB).coef;
            } else {
                cv = lane < A ? a.dz[(size_t)row * A + lane] : (lane == A ? a.dv[row] : 0.f);
            }
            const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(cv), A));
            float4 acc = make_float4(d * wv.x, d * wv.y, d * wv.z, d * wv.w);
#pragma unroll
            for (int k = 0; k < AMAX; ++k)
                if (k < A) {
                    const float g = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(cv), k));
                    acc.x += g * w[k].x; acc.y += g * w[k].y; acc.z += g * w[k].z; acc.w += g * w[k].w;
                }
            acc.x = hv.x > 0.f ? acc.x : 0.f; acc.y = hv.y > 0.f ? acc.y : 0.f;
            acc.z = hv.z > 0.f ? acc.z : 0.f; acc.w = hv.w > 0.f ? acc.w : 0.f;
            if (a.dh_b) {
                auto bf = [](float f) { __bf16 b = (__bf16)f; return (unsigned)__builtin_bit_cast(unsigned short, b); };
                *reinterpret_cast<uint2*>(a.dh_b + (size_t)row * F + j) = make_uint2(bf(acc.x) | (bf(acc.y) << 16), bf(acc.z) | (bf(acc.w) << 16));
            } else {
                *reinterpret_cast<float4*>(a.dh + (size_t)row * F + j) = acc;
            }
        }
        return;
    }
    constexpr int RQ = FUSED ? 4 : 8;               // rows of a wave in flight
    __shared__ float part[4][AMAX + 1][64];
    __shared__ float partb[4][AMAX + 1];
    __shared__ float lossp[4][3];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wb = blockIdx.x - a.n_dh, fx = F / 64, fxi = wb % fx, c = wb / fx, K1 = A + 1;
    const int j = fxi * 64 + lane;
    const int r0 = c * a.rows_per_chunk, r1 = min(rows, r0 + a.rows_per_chunk);      // a trailing chunk may be empty: zeros
    float acc[AMAX + 1], accb[AMAX + 1];
#pragma unroll
    for (int k = 0; k <= AMAX; ++k) { acc[k] = 0.f; accb[k] = 0.f; }
    float s_pl = 0.f, s_h = 0.f, s_vl = 0.f;
    for (int r = r0 + wave; r < r1; r += 4 * RQ) {     // RQ of this wave's rows in flight
        float hv[RQ], cv[RQ];                          // cv: lane k holds coefficient k of the row (zero past the chunk)
        RowIn in[RQ];
#pragma unroll
        for (int q = 0; q < RQ; ++q) {
            const int rr = r + 4 * q;
            hv[q] = a.h[(size_t)min(rr, r1 - 1) * F + j];
            if constexpr (FUSED) in[q] = row_load(a.loss, min(rr, r1 - 1), lane);
            else cv[q] = (rr < r1 && lane < K1) ? (lane < A ? a.dz[(size_t)rr * A + lane] : a.dv[rr]) : 0.f;
        }
        if constexpr (FUSED) {
#pragma unroll
            for (int q = 0; q < RQ; ++q) {
                const int rr = r + 4 * q;
                cv[q] = 0.f;
                if (rr < r1) {                         // uniform in the wavefront
                    const RowOut o = row_compute(a.loss, in[q], rr, lane, gamma, beta, cvc, invB);
                    cv[q] = o.coef;
                    if (fxi == 0) {
                        s_pl += o.pl; s_h += o.H; s_vl += o.vl;
                        if (lane < A) a.loss.dz[(size_t)rr * A + lane] = o.coef;
                        if (lane == A) a.loss.dv[rr] = o.coef;
                        if (lane == 0) a.loss.returns[rr] = o.R;
                    }
                }
            }
        }
#pragma unroll
        for (int q = 0; q < RQ; ++q) {
#pragma unroll
            for (int k = 0; k <= AMAX; ++k)
                if (k < K1) {
                    const float g = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(cv[q]), k));
                    acc[k] += g * hv[q]; accb[k] += g;
                }
        }
    }
#pragma unroll
    for (int k = 0; k <= AMAX; ++k)
        if (k < K1) { part[wave][k][lane] = acc[k]; if (lane == 0) partb[wave][k] = accb[k]; }
    if (FUSED && lane == 0) { lossp[wave][0] = s_pl * invB; lossp[wave][1] = s_h * invB; lossp[wave][2] = s_vl * invB; }
    __syncthreads();
    for (int e = tid; e < K1 * 64; e += 256) {
        const int k = e / 64, l = e % 64;
        a.pw[((size_t)c * K1 + k) * F + fxi * 64 + l] = ((part[0][k][l] + part[1][k][l]) + part[2][k][l]) + part[3][k][l];
    }
    if (fxi == 0 && tid < K1) a.pb[c * K1 + tid] = ((partb[0][tid] + partb[1][tid]) + partb[2][tid]) + partb[3][tid];
    // the chunk's share of the three loss means (each carries the 1/B of the batch mean)
    if (FUSED && fxi == 0 && tid < 3) a.loss.loss_partials[c * 4 + tid] = ((lossp[0][tid] + lossp[1][tid]) + lossp[2][tid]) + lossp[3][tid];
}

bool heads_bwd_fuses_loss(int rows, int A, int T, int F) {
    return rows < 1024 && A <= 32 && T <= 64 && (F / 4) % 64 == 0 && 256 % (F / 4) == 0;
}

template <bool FUSED> static void launch_heads_bwd_rows(hipStream_t s, const dim3 grid, const HeadsBwdArgs& a) {
    if (a.A <= 8) launch_k((heads_bwd_rows_kernel<8, FUSED>), grid, dim3(256), s, a);
    else if (a.A <= 18) launch_k((heads_bwd_rows_kernel<18, FUSED>), grid, dim3(256), s, a);
    else launch_k((heads_bwd_rows_kernel<32, FUSED>), grid, dim3(256), s, a);
}

hipError_t heads_bwd(hipStream_t s, int F, int A, int rows, int n_chunk, const float* dz, const float* dv, const float* pi_w,
                     const float* v_w, const float* h, float* dh, bf16_t* dh_b, float* pw, float* pb, const LossArgs* fused_loss) {
    if (rows <= 0 || n_chunk <= 0 || F % 256 != 0) return hipErrorInvalidValue;
    const int n_dh = (rows * (F / 4) + 255) / 256;
    const int rpc = (rows + n_chunk - 1) / n_chunk;
    if (fused_loss) {
        const LossArgs& la = *fused_loss;
        if (!heads_bwd_fuses_loss(rows, A, la.T, F) || la.A != A || la.T * la.n_e != rows) return hipErrorInvalidValue;
        const int rpi = 256 / (F / 4);                       // one pass of a dh block: a row per wave or pair of waves
        const int n_dh_rows = (rows + rpi - 1) / rpi;
        HeadsBwdArgs a{F, A, rows, n_dh_rows, rpi, rpc, nullptr, nullptr, pi_w, v_w, h, dh, dh_b, pw, pb, la};
        launch_heads_bwd_rows<true>(s, dim3(n_dh_rows + (F / 64) * n_chunk), a);
        return hipGetLastError();
    }
    if (rows >= 1024 && A <= 32 && (F / 4) % 64 == 0 && 256 % (F / 4) == 0) {            // large batches: h is read once
        const int rpi = 256 / (F / 4);                       // rows a dh block works on at once
        int rpd = rows / 512;                                // enough dh blocks to fill the chip, at most 32 rows each
        rpd = rpd > 32 ? 32 : rpd;
        rpd = (rpd + rpi - 1) / rpi * rpi;
        const int n_dh = (rows + rpd - 1) / rpd;
        HeadsBwdArgs a{F, A, rows, n_dh, rpd, rpc, dz, dv, pi_w, v_w, h, dh, dh_b, pw, pb, LossArgs{}};
        launch_heads_bwd_rows<false>(s, dim3(n_dh + (F / 64) * n_chunk), a);
        return hipGetLastError();
    }
    launch_k(heads_bwd_kernel, dim3(n_dh + (F / 256) * (A + 1) * n_chunk), dim3(256), s, F, A, rows, n_dh, rpc, dz, dv, pi_w, v_w, h,
             dh, dh_b, pw, pb);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ gradient reduction + norm
// Sum over the 256 threads of a block (every thread gets it): within the waves with DPP moves, then
// the four wave sums through LDS in wave order; two barriers (a tree through LDS took nine).
__device__ __forceinline__ float block_sum_256(float v, float* red) {
    const float w = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
    __syncthreads();
    const float r = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return r;
}

// Sums the split partial gradients in a fixed order (bit-stable from run to run), writes the
// gradient arena and one partial sum of squares per block.  Four consecutive arena elements per
// thread (tensors start at multiples of 64 floats, so the four belong to one tensor), 16-byte loads
// where the partial buffer allows.  Split q goes to accumulator q mod 8 in ascending q, the eight
// are added as a tree; 8 or 16 loads are issued before the first addition (a first-layer weight gradient
// has 60+ splits: issued one after the other they were the critical path of the whole kernel).
__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ __forceinline__ float add4(float a, float b) { return a + b; }
template <class V> __device__ __forceinline__ V zero_v();
template <> __device__ __forceinline__ float zero_v<float>() { return 0.f; }
template <> __device__ __forceinline__ float4 zero_v<float4>() { return make_float4(0.f, 0.f, 0.f, 0.f); }

template <class V, int R>
__device__ __forceinline__ void sum_rounds(const float* p, size_t st, int ns, V (&acc)[8]) {
    for (int q = 0; q < ns; q += R) {
        V v[R];
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = *reinterpret_cast<const V*>(p + (size_t)min(q + r, ns - 1) * st);   // clamped: ignored below
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r & 7] = add4(acc[r & 7], q + r < ns ? v[r] : zero_v<V>());
    }
}
template <class V>
__device__ __forceinline__ V sum_splits(const float* p, size_t st, int ns) {
    V acc[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) acc[r] = zero_v<V>();
    if (ns == 1) return *reinterpret_cast<const V*>(p);
    if (ns > 8) sum_rounds<V, 16>(p, st, ns, acc);
    else sum_rounds<V, 8>(p, st, ns, acc);
    return add4(add4(add4(acc[0], acc[1]), add4(acc[2], acc[3])), add4(add4(acc[4], acc[5]), add4(acc[6], acc[7])));
}

__global__ __launch_bounds__(256) void grad_reduce_norm_kernel(const GradSegments seg, float* grads, float* block_ss) {
    __shared__ float red[256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int sidx = 0;
    for (int q = 1; q < seg.n; ++q) if ((int)blockIdx.x >= seg.blk_off[q]) sidx = q;      // uniform: scalar loads of the arguments
    const int lb = blockIdx.x - seg.blk_off[sidx];
    const int count = seg.count[sidx], padded = seg.padded[sidx], ns = seg.n_split[sidx];
    const size_t st = seg.stride[sidx];
    float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
    bool owner = true;
    int local;
    if (seg.lanes[sidx] == 1) {
        local = (lb * 256 + tid) * 4;
        if (local < padded) {
            const float* p = seg.partial[sidx] + local;
            if (local + 3 < count && (reinterpret_cast<uintptr_t>(p) & 15) == 0 && (st & 3) == 0) {
                g = sum_splits<float4>(p, st, ns);
            } else {
                if (local < count) g.x = sum_splits<float>(p, st, ns);
                if (local + 1 < count) g.y = sum_splits<float>(p + 1, st, ns);
                if (local + 2 < count) g.z = sum_splits<float>(p + 2, st, ns);
                if (local + 3 < count) g.w = sum_splits<float>(p + 3, st, ns);
            }
        }
    } else {
        // eight consecutive quads per wave and split lane: lane = j * 8 + quad (128 contiguous bytes per split lane)
        const int j = lane >> 3;
        local = ((lb * 4 + wave) * 8 + (lane & 7)) * 4;
        owner = j == 0;
        if (local < count) {                                      // count is a multiple of 4 in these segments
            const float* p = seg.partial[sidx] + local;
            for (int q = j; q < ns; q += 8 * 16) {
                float4 v[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) v[r] = *reinterpret_cast<const float4*>(p + (size_t)min(q + 8 * r, ns - 1) * st);   // clamped: ignored below
#pragma unroll
                for (int r = 0; r < 16; ++r) if (q + 8 * r < ns) g = add4(g, v[r]);
            }
        }
        // lanes j and j^1, then pairs, then halves: ((0+1)+(2+3)) + ((4+5)+(6+7))
#pragma unroll
        for (int o = 8; o < 64; o <<= 1) {
            g.x += __shfl_xor(g.x, o); g.y += __shfl_xor(g.y, o); g.z += __shfl_xor(g.z, o); g.w += __shfl_xor(g.w, o);
        }
    }
    float ss = 0.f;
    if (owner && local < padded) {
        float* dst = grads + seg.off[sidx] + local;
        if (seg.partial[sidx] + local != dst) *reinterpret_cast<float4*>(dst) = g;      // an unsplit gradient may already be in place
        ss = (g.x * g.x + g.y * g.y) + (g.z * g.z + g.w * g.w);
    }
    const float tot = block_sum_256(ss, red);
    if (tid == 0) block_ss[blockIdx.x] = tot;
}

hipError_t grad_reduce_norm(hipStream_t s, const GradSegments& seg, float* grads, float* block_ss) {
    const int blocks = seg.blk_off[seg.n];
    if (blocks < 1) return hipErrorInvalidValue;
    launch_k(grad_reduce_norm_kernel, dim3(blocks), dim3(256), s, seg, grads, block_ss);
    return hipGetLastError();
}

// An fp32 number as three bf16 numbers whose sum it is: its 24 significand bits cut into 8 + 8 + 8
// by truncation (both residuals are exact).  Element (k, c) of weight matrix l goes to its place in
// the fragment order described at WeightSplits.
__device__ __forceinline__ void store_split3(float w, int c, int k, bf16_t* parts, int K, int plane) {
    const uint32_t hb = __float_as_uint(w) & 0xffff0000u;
    const float r1 = w - __uint_as_float(hb);
    const uint32_t mb = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(mb);
    const int at = (((c >> 5) * (K >> 4) + (k >> 4)) * 64 + ((k >> 3) & 1) * 32 + (c & 31)) * 8 + (k & 7);
    parts[at] = (bf16_t)(hb >> 16);
    parts[plane + at] = (bf16_t)(mb >> 16);
    parts[2 * plane + at] = (bf16_t)(__float_as_uint(r2) >> 16);
}

// the same for two numbers, parts packed (a in the low half)
__device__ __forceinline__ void split3_pack(float a, float b, unsigned& hi, unsigned& mid, unsigned& lo) {
    const uint32_t ah = __float_as_uint(a) & 0xffff0000u, bh = __float_as_uint(b) & 0xffff0000u;
    const float a1 = a - __uint_as_float(ah), b1 = b - __uint_as_float(bh);
    const uint32_t am = __float_as_uint(a1) & 0xffff0000u, bm = __float_as_uint(b1) & 0xffff0000u;
    const float a2 = a1 - __uint_as_float(am), b2 = b1 - __uint_as_float(bm);
    hi = (ah >> 16) | bh;
    mid = (am >> 16) | bm;
    lo = (__float_as_uint(a2) >> 16) | (__float_as_uint(b2) & 0xffff0000u);
}

// Every weight matrix of ws from the fp32 arena; one thread per element of the padded matrices
// (columns C .. next multiple of 32 are written as zeros).
__global__ __launch_bounds__(256) void split_weights_kernel(const WeightSplits ws, const float* theta) {
    int i = blockIdx.x * 256 + threadIdx.x;
    for (int l = 0; l < ws.n; ++l) {
        const int plane = ws.plane(l);
        if (i < plane) {
            const int cp = plane / ws.K[l], k = i / cp, c = i % cp;
            store_split3(c < ws.C[l] ? theta[ws.off[l] + k * ws.C[l] + c] : 0.f, c, k, ws.dst[l], ws.K[l], plane);
            return;
        }
        i -= plane;
    }
}
hipError_t split_weights(hipStream_t s, const WeightSplits& ws, const float* theta) {
    int total = 0;
    for (int l = 0; l < ws.n; ++l) {
        if (ws.K[l] % 16 != 0 || ws.off[l] % 4 != 0 || (ws.K[l] * ws.C[l]) % 4 != 0 || !ws.dst[l]) return hipErrorInvalidValue;
        total += ws.plane(l);
    }
    if (total == 0) return hipSuccess;
    launch_k(split_weights_kernel, dim3((total + 255) / 256), dim3(256), s, ws, theta);
    return hipGetLastError();
}

// Global-norm clip (scale = min(1, c/||g||)) fused with RMSProp, epsilon inside the root:
//   g2 <- alpha g2 + (1-alpha) (s g)^2 ;  theta <- theta - lr (s g) / sqrt(g2 + eps).
// Every block re-derives the norm from the per-block partial sums (same order everywhere).
// The updated weights of the matrices listed in ws are also written in the forms the next forward and
// backward pass read (three bf16 parts in the fp32 configuration, bf16 copies in the bf16 one).
__global__ __launch_bounds__(256) void rmsprop_update_kernel(int n4, float4* theta, float4* g2, const float4* grads,
                                                             const float* block_ss, int n_ss, const float* hp,
                                                             const float* loss_partials, int n_loss_blocks,
                                                             StatsOut* stats_a, StatsOut* stats_b,
                                                             const WeightMirrors ws, int ws_blocks) {
    __shared__ float red[256];
    float part = 0.f;
    for (int q = threadIdx.x; q < n_ss; q += 256) part += block_ss[q];
    const float tot = block_sum_256(part, red);
    const float norm = sqrtf(tot);
    const float clip = hp[HP_CLIP], lr = hp[HP_LR], alpha = hp[HP_ALPHA], eps = hp[HP_EPS];
    const float scale = norm > clip ? clip / norm : 1.0f;
    const float oma = 1.0f - alpha;
    // The matrices of ws are updated by the first ws_blocks workgroups, one thread per (eight
    // consecutive k, column): lanes along the columns read and write whole rows, and a thread holds
    // exactly the eight values of one 16-byte slot of a part buffer or of a k-contiguous bf16 copy.
    if ((int)blockIdx.x < ws_blocks) {
        int u = blockIdx.x * 256 + threadIdx.x;
        for (int l = 0; l < ws.n; ++l) {
            const int C = ws.C[l], K = ws.K[l], units = (K >> 3) * C;
            if (u < units) {
                const int k8 = u / C, c = u % C;
                float* th = reinterpret_cast<float*>(theta); float* v2 = reinterpret_cast<float*>(g2);
                const float* gr = reinterpret_cast<const float*>(grads);
                float gv[8], vv[8], tv[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int at = ws.off[l] + (k8 * 8 + j) * C + c;
                    gv[j] = gr[at]; vv[j] = v2[at]; tv[j] = th[at];
                }
                unsigned hi[4], mid[4], lo[4];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int at = ws.off[l] + (k8 * 8 + j) * C + c;
                    const float g = gv[j] * scale;
                    vv[j] = alpha * vv[j] + oma * g * g;
                    tv[j] -= lr * g / sqrtf(vv[j] + eps);
                    v2[at] = vv[j]; th[at] = tv[j];
                }
                if (ws.split[l]) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) split3_pack(tv[2 * j], tv[2 * j + 1], hi[j], mid[j], lo[j]);
                    const int plane = ws.plane(l);
                    bf16_t* d = ws.split[l] + (size_t)((((c >> 5) * (K >> 4) + (k8 >> 1)) * 64 + (k8 & 1) * 32 + (c & 31)) * 8);
                    *reinterpret_cast<uint4*>(d) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
                    *reinterpret_cast<uint4*>(d + plane) = make_uint4(mid[0], mid[1], mid[2], mid[3]);
                    *reinterpret_cast<uint4*>(d + 2 * plane) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
                }
                auto bf = [](float f) { __bf16 b = (__bf16)f; return (unsigned)__builtin_bit_cast(unsigned short, b); };
                for (int d = 0; d < 2; ++d) {
                    bf16_t* dst = ws.copy[l][d];
                    if (!dst) continue;
                    const int mode = ws.mode[l][d];
                    if (mode == 0 || mode == 3) {          // k-contiguous: one 16-byte store
                        const uint4 w = make_uint4(bf(tv[0]) | (bf(tv[1]) << 16), bf(tv[2]) | (bf(tv[3]) << 16),
                                                   bf(tv[4]) | (bf(tv[5]) << 16), bf(tv[6]) | (bf(tv[7]) << 16));
                        const size_t at = mode == 0 ? (size_t)c * K + k8 * 8 : (size_t)k8 * 256 + c * 8;
                        *reinterpret_cast<uint4*>(dst + at) = w;
                    } else if (mode == 1) {                // the matrix as it is: lanes write consecutive columns
#pragma unroll
                        for (int j = 0; j < 8; ++j) dst[(size_t)(k8 * 8 + j) * C + c] = (bf16_t)bf(tv[j]);
                    } else {                               // [ci][tap][co]: eight consecutive k are eight channels of one tap
                        const int cin = ws.cin[l], T = K / cin, tap = (k8 * 8) / cin, ci0 = (k8 * 8) % cin;
#pragma unroll
                        for (int j = 0; j < 8; ++j) dst[((size_t)(ci0 + j) * T + tap) * C + c] = (bf16_t)bf(tv[j]);
                    }
                }
                break;
            }
            u -= units;
        }
        return;
    }
    auto update = [&](int i, float4 g, float4 v, float4 t) __attribute__((always_inline)) {
        for (int l = 0; l < ws.n; ++l) {                           // offsets and sizes are multiples of 4
            const int e0 = i * 4 - ws.off[l];
            if (e0 >= 0 && e0 < ws.K[l] * ws.C[l]) return;         // updated above
        }
        g.x *= scale; g.y *= scale; g.z *= scale; g.w *= scale;
        v.x = alpha * v.x + oma * g.x * g.x; v.y = alpha * v.y + oma * g.y * g.y;
        v.z = alpha * v.z + oma * g.z * g.z; v.w = alpha * v.w + oma * g.w * g.w;
        t.x -= lr * g.x / sqrtf(v.x + eps); t.y -= lr * g.y / sqrtf(v.y + eps);
        t.z -= lr * g.z / sqrtf(v.z + eps); t.w -= lr * g.w / sqrtf(v.w + eps);
        g2[i] = v; theta[i] = t;
    };
    const int stride = (gridDim.x - ws_blocks) * 256;
    int i = (blockIdx.x - ws_blocks) * 256 + threadIdx.x;
    for (; i + stride < n4; i += 2 * stride) {                    // two elements' loads in flight
        const float4 ga = grads[i], va = g2[i], ta = theta[i];
        const float4 gb = grads[i + stride], vb = g2[i + stride], tb = theta[i + stride];
        update(i, ga, va, ta);
        update(i + stride, gb, vb, tb);
    }
    if (i < n4) update(i, grads[i], g2[i], theta[i]);
    if ((int)blockIdx.x == ws_blocks && threadIdx.x < 64) {
        // lane l adds the partials l, l + 64, ... in ascending order, then the lanes are added: a fixed order
        float pl = 0.f, en = 0.f, vl = 0.f;
        for (int b = threadIdx.x; b < n_loss_blocks; b += 64) { pl += loss_partials[b * 4]; en += loss_partials[b * 4 + 1]; vl += loss_partials[b * 4 + 2]; }
        pl = wave_sum(pl); en = wave_sum(en); vl = wave_sum(vl);
        if (threadIdx.x != 0) return;
        StatsOut st;
        // each block's partial already carries the 1/B of the batch mean
        st.policy_loss = pl; st.entropy = en; st.value_loss = vl;
        st.total_loss = pl - hp[HP_BETA] * en + hp[HP_VCOEF] * vl;
        st.grad_norm = norm; st.clip_scale = scale;
        st.nonfinite = (isfinite(st.total_loss) && isfinite(norm)) ? 0 : 1;
        if (stats_a) *stats_a = st;
        if (stats_b) *stats_b = st;
    }
}

hipError_t rmsprop_update(hipStream_t s, int p_int, float* theta, float* g2, const float* grads, const float* block_ss,
                          int n_ss, const float* hp, const float* loss_partials, int n_loss_blocks, StatsOut* stats_a, StatsOut* stats_b,
                          const WeightMirrors& ws) {
    const int n4 = p_int / 4;
    int blocks = (n4 + 255) / 256;
    if (blocks > 512) blocks = 512;       // grid-stride loop: fewer, longer-lived workgroups
    int units = 0;
    for (int l = 0; l < ws.n; ++l) units += (ws.K[l] / 8) * ws.C[l];
    const int ws_blocks = (units + 255) / 256;
    launch_k(rmsprop_update_kernel, dim3(ws_blocks + blocks), dim3(256), s, n4, (float4*)theta, (float4*)g2,
                       (const float4*)grads, block_ss, n_ss, hp, loss_partials, n_loss_blocks, stats_a, stats_b,
                       ws, ws_blocks);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ Philox4x32-10
// Salmon, Moraes, Dror, Shaw (SC'11).  Same function on host (parameter init) and device.
__host__ __device__ inline void philox_round(uint32_t& c0, uint32_t& c1, uint32_t& c2, uint32_t& c3, uint32_t k0, uint32_t k1) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
}
__host__ __device__ inline void philox_block(uint64_t ctr, uint64_t key, uint32_t out[4]) {
    uint32_t c0 = (uint32_t)ctr, c1 = (uint32_t)(ctr >> 32), c2 = 0, c3 = 0;
    uint32_t k0 = (uint32_t)key, k1 = (uint32_t)(key >> 32);
    for (int r = 0; r < 10; ++r) {
        philox_round(c0, c1, c2, c3, k0, k1);
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        philox_round(c0, c1, c2, c3, k0, k1);
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__global__ __launch_bounds__(256) void fill_uniforms_kernel(uint64_t seed, uint64_t offset, float* out, size_t n) {
    const size_t b = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (b * 4 >= n) return;
    uint32_t w[4];
    philox_block(offset + b, seed, w);
    for (int i = 0; i < 4; ++i)
        if (b * 4 + i < n) out[b * 4 + i] = (float)(w[i] >> 8) * (1.0f / 16777216.0f);
}

hipError_t fill_uniforms(hipStream_t s, uint64_t seed, uint64_t offset, float* out, size_t n) {
    if (n == 0) return hipSuccess;
    const size_t blocks = ((n + 3) / 4 + 255) / 256;
    launch_k(fill_uniforms_kernel, dim3((unsigned)blocks), dim3(256), s, seed, offset, out, n);
    return hipGetLastError();
}

// Holds the stream busy for about `us` microseconds (bounded spin on the 100 MHz wall clock) so that
// the launches that follow are already queued when the GPU reaches them: used only by the per-kernel
// timing mode, whose event pairs would otherwise also measure the host's launch rate.
__global__ void delay_kernel(unsigned us) {
    const unsigned long long t0 = wall_clock64();
    const unsigned long long ticks = (unsigned long long)us * 100ull;
    for (int it = 0; it < 2000000; ++it) {             // hard bound: the kernel always exits
        if (wall_clock64() - t0 >= ticks) break;
        __builtin_amdgcn_s_sleep(32);
    }
}
hipError_t delay_us(hipStream_t s, unsigned us) {
    launch_k(delay_kernel, dim3(1), dim3(1), s, us);
    return hipGetLastError();
}

}  // namespace paac
