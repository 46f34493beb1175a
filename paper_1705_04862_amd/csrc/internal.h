// Internal interfaces between the translation units of libpaac (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

namespace paac {

// Every kernel of the library is launched through launch_k.  In the per-kernel timing mode the
// caller sets tl_prof around one launch; the launch then carries a start/stop event pair that is
// stamped with the kernel's own begin and end on the GPU (independent of the host's launch rate).
struct ProfEvents { hipEvent_t start, stop; };
extern thread_local ProfEvents tl_prof;
template <class K, class... Args>
inline void launch_k(K kernel, dim3 grid, dim3 block, hipStream_t s, Args... args) {
    if (tl_prof.start) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, tl_prof.start, tl_prof.stop, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, 0, s, args...);
}
// the same with `lds_bytes` of dynamic LDS
template <class K, class... Args>
inline void launch_k_lds(K kernel, dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t s, Args... args) {
    if (tl_prof.start) hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, s, tl_prof.start, tl_prof.stop, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, lds_bytes, s, args...);
}

// Static description of one of the two networks (Experiments: arch_nips, arch_nature).
struct ConvDesc { int cin, h, w, ks, st, cout, ho, wo, kk; };
struct NetDesc {
    int arch, n_conv;
    ConvDesc conv[3];
    int flat, fc, n_actions;
};
NetDesc make_net(int arch, int n_actions);

// How one contraction is split over workgroups along its reduction dimension.
struct Split { int n; int k_per; };
Split plan_split(int k_total, int tiles, int granule, int target_wgs);

// ---- dense layers (layers.hip); all activations are NHWC, weights are [K][c_out] ----
// conv forward + bias + ReLU over `ns` samples.  Layer 0 reads uint8 NCHW states (k = c,ky,kx),
// later layers read float NHWC (k = ky,kx,c).
hipError_t conv_fwd(hipStream_t s, int arch, int layer, const void* in, const float* W, const float* b,
                    float* out, int ns);
// dX = dY (*) W^T in gather form, multiplied by ReLU'(act_in); layer >= 1.
hipError_t conv_dgrad(hipStream_t s, int arch, int layer, const float* dy, const float* W,
                      const float* act_in, float* dx, int ns);
// partial_w[split][K][c_out], partial_b[split][c_out]; rows of the reduction are output positions.
int conv_wgrad_tiles(int arch, int layer);
hipError_t conv_wgrad(hipStream_t s, int arch, int layer, const void* in, const float* dy, float* partial_w,
                      float* partial_b, int ns, Split sp);
// fc forward: partial[split][ns][fc] = x[ns][flat(k-range)] . W[flat][fc]   (no bias, no ReLU)
int fc_fwd_tiles(int arch, int ns);
int fc_fwd_target_wgs(int ns);
hipError_t fc_fwd(hipStream_t s, int arch, const float* x, const float* W, float* partial, int ns, Split sp);
// dx[ns][flat] = (dh[ns][fc] . W^T) * 1[act > 0]
hipError_t fc_dgrad(hipStream_t s, int arch, const float* dh, const float* W, const float* act, float* dx, int ns);
// partial_w[split][flat][fc] = x^T . dh over a range of samples; partial_b[split][fc] = column sums of dh
int fc_wgrad_tiles(int arch);
hipError_t fc_wgrad(hipStream_t s, int arch, const float* x, const float* dh, float* partial_w, float* partial_b,
                    int ns, Split sp);
// fused data + weight gradient of one layer (one launch)
hipError_t conv_bwd(hipStream_t s, int arch, int layer, const float* act_in, const float* dy, const float* W, float* dx,
                    float* pw, float* pb, int ns, Split sp);
hipError_t fc_bwd(hipStream_t s, int arch, const float* x, const float* dh, const float* W, float* dx, float* pw, float* pb,
                  int ns, Split sp);

// ---- the same layers with bf16 operands (layers_bf16.hip): bf16 NHWC activations, bf16 weight copies
// (forward copy Wt[c_out][K], data-gradient copy Wd[c_in][ky,kx][c_out]; fc: Wt[fc][flat], Wc[flat][fc]),
// fp32 bias, fp32 partial sums and gradients ----
typedef unsigned short bf16_t;
hipError_t conv_fwd_bf16(hipStream_t s, int arch, int layer, const void* in, const bf16_t* Wt, const float* b,
                         bf16_t* out, int ns);
hipError_t conv_dgrad_bf16(hipStream_t s, int arch, int layer, const bf16_t* dy, const bf16_t* Wd, const bf16_t* act_in,
                           bf16_t* dx, int ns);
int conv_wgrad_tiles_bf16(int arch, int layer);
hipError_t conv_wgrad_bf16(hipStream_t s, int arch, int layer, const void* in, const bf16_t* dy, float* partial_w,
                           float* partial_b, int ns, Split sp);
int fc_fwd_tiles_bf16(int arch, int ns);
hipError_t fc_fwd_bf16(hipStream_t s, int arch, const bf16_t* x, const bf16_t* Wt, float* partial, int ns, Split sp);
hipError_t fc_dgrad_bf16(hipStream_t s, int arch, const bf16_t* dh, const bf16_t* Wc, const bf16_t* act, bf16_t* dx, int ns);
int fc_wgrad_tiles_bf16(int arch);
hipError_t fc_wgrad_bf16(hipStream_t s, int arch, const bf16_t* x, const bf16_t* dh, float* partial_w, float* partial_b,
                         int ns, Split sp);
constexpr int kMaxCopies = 8;
struct WeightCopies {            // see make_bf16_weights_kernel for the modes
    int n, total;
    bf16_t* dst[kMaxCopies]; int start[kMaxCopies], src_off[kMaxCopies], K[kMaxCopies], C[kMaxCopies], cin[kMaxCopies], mode[kMaxCopies];
};
// fp32 configuration: convolution weights W[K][C] also kept as three bf16 parts whose sum they are, in
// the order in which the lanes of the exact-operand kernels read their MFMA B fragments:
//   dst[part][C/32 rounded up][K/16][64 lanes = (k%16)/8 * 32 + c%32][8 = k%8]   (columns past C are zero)
struct WeightSplits {
    int n;
    int off[3], K[3], C[3];      // arena offset (floats, multiple of 4), rows (multiple of 16), columns
    bf16_t* dst[3];
    __host__ __device__ int plane(int l) const { return (C[l] + 31) / 32 * 32 * K[l]; }
};
hipError_t split_weights(hipStream_t s, const WeightSplits& ws, const float* theta);
// What the optimiser writes besides theta when it updates weight matrix W[K][C] (K a multiple of 8):
// the three bf16 parts (fp32 configuration) and / or up to two bf16 copies in the layouts of
// make_bf16_weights_kernel (bf16 configuration), so that no separate pass over the weights follows.
constexpr int kMaxMirrors = 4;
struct WeightMirrors {
    int n;
    int off[kMaxMirrors], K[kMaxMirrors], C[kMaxMirrors], cin[kMaxMirrors];
    bf16_t* split[kMaxMirrors];                 // parts in fragment order (see WeightSplits), or null
    bf16_t* copy[kMaxMirrors][2];               // bf16 copies, or null
    int mode[kMaxMirrors][2];
    __host__ __device__ int plane(int l) const { return (C[l] + 31) / 32 * 32 * K[l]; }
};
// first convolution of the fp32 path from the three bf16 parts of its weights, fp32 NHWC output
hipError_t conv1_fwd_exact(hipStream_t s, int arch, const uint8_t* x, const bf16_t* w_parts, const float* b, float* out, int ns);
// layers 1.. of the fp32 path, one sample per workgroup, from the parts of weights and activations
hipError_t conv_fwd_exact(hipStream_t s, int arch, int layer, const float* in, const bf16_t* w_parts, const float* b, float* out, int ns);
// all convolutions of the fp32 path in one launch, one workgroup per sample; ns <= trunk_fwd_exact_max()
int trunk_fwd_exact_max();
hipError_t trunk_fwd_exact(hipStream_t s, int arch, const uint8_t* x, const bf16_t* const* w_parts, const float* const* b, float* const* out, int ns);
// first convolution's weight gradient from the image; dy fp32 (exact) or bf16; writes n_wgs partials [256][cout] / [cout]
hipError_t conv1_wgrad_direct(hipStream_t s, int arch, bool exact, const uint8_t* x, const void* dy, float* pw, float* pb, int ns, int n_wgs);
hipError_t make_bf16_weights(hipStream_t s, const WeightCopies& w, const float* theta);
// bf16 configuration: partial sums (= workgroups) of the per-sample weight-gradient kernel of a layer,
// 0 where the tiled GEMM with its split plan is used; conv_wgrad_bf16 takes them as Split{n, 0}
int conv_wgrad_direct_wgs(int arch, int layer, int ns);

// ---- small kernels (small_kernels.hip) ----
struct HeadsArgs {
    const float* fc_partial; int n_split; size_t split_stride;   // [split][rows][F]
    const float* fc_b; const float* pi_w; const float* pi_b; const float* v_w; const float* v_b;
    int rows, A;
    float* h_out;          // [rows][F] or null
    float* logits_out;     // [rows][A] or null
    float* values_out;     // [rows] or null
    float* values_copy;    // [rows] or null: a second destination for the values
    const float* uniforms; // select mode when non-null
    int32_t* actions_out;  // [rows]
    float* probs_out;      // [rows][A] or null
    int algorithm;         // ALG_*: how the action is drawn from the head outputs
    float epsilon;         // exploration rate of ALG_NSTEP_Q
};
hipError_t heads_fwd(hipStream_t s, int F, const HeadsArgs& a);

struct LossArgs {
    const float* logits; const float* values;           // [(T+1) n_e][A], [(T+1) n_e]
    const int32_t* actions; const float* rewards; const uint8_t* dones;
    const float* hp;                                     // device hyper-parameters (HP_* indices)
    int T, n_e, A;
    float* returns; float* dz; float* dv;                // [T n_e], [T n_e][A], [T n_e]
    float* loss_partials;                                // [blocks][4]
    int algorithm;                                       // ALG_*
};
int loss_blocks(int n_e);
hipError_t returns_loss(hipStream_t s, const LossArgs& a);

// head backward in one launch: dh (fp32, or bf16 when dh_b is non-null) and the split weight gradients
// partial_w[chunk][A+1][F] (row A = value head), partial_b[chunk][A+1]
hipError_t heads_bwd(hipStream_t s, int F, int A, int rows, int n_chunk, const float* dz, const float* dv, const float* pi_w,
                     const float* v_w, const float* h, float* dh, bf16_t* dh_b, float* partial_w, float* partial_b, const LossArgs* fused_loss);
// whether heads_bwd takes the returns + loss work into its own launch: then fused_loss is given,
// returns_loss is not launched, and loss_partials holds one entry per chunk of rows (n_chunk of them)
bool heads_bwd_fuses_loss(int rows, int A, int T, int F);

enum { ALG_ACTOR_CRITIC = 0, ALG_NSTEP_Q = 1 };
enum { HP_GAMMA = 0, HP_BETA, HP_VCOEF, HP_LR, HP_ALPHA, HP_EPS, HP_CLIP, HP_COUNT = 8 };

constexpr int kMaxSeg = 12;
// Gradient reduction: one segment per parameter tensor.  A workgroup of the reduction belongs to one
// segment; a thread owns four consecutive elements and, in segments with many splits, one of eight
// split lanes (lanes[s] = 8: the splits q = j, j + 8, ... go to lane j, the eight lanes are added as
// a tree), so that a tensor with hundreds of partial sums is not summed by a handful of threads.
struct GradSegments {
    int n;
    const float* partial[kMaxSeg]; int n_split[kMaxSeg]; size_t stride[kMaxSeg];
    int count[kMaxSeg]; int off[kMaxSeg]; int padded[kMaxSeg];
    int lanes[kMaxSeg]; int blk_off[kMaxSeg + 1];         // filled by plan_reduce_blocks
};
inline int norm_blocks_cap(int p_int) { return p_int / 128 + 2 * kMaxSeg; }   // upper bound of the reduction's workgroups
inline int plan_reduce_blocks(GradSegments& g) {
    int blocks = 0;
    for (int s = 0; s < g.n; ++s) {
        const bool vec = (reinterpret_cast<uintptr_t>(g.partial[s]) & 15) == 0 && (g.stride[s] & 3) == 0 && (g.count[s] & 3) == 0;
        g.lanes[s] = (vec && g.n_split[s] >= 32) ? 8 : 1;
        g.blk_off[s] = blocks;
        blocks += (g.padded[s] / 4 * g.lanes[s] + 255) / 256;
    }
    g.blk_off[g.n] = blocks;
    return blocks;
}
// grads[i] = sum over splits of the partial gradients; block_ss[workgroup] = partial sums of g^2
hipError_t grad_reduce_norm(hipStream_t s, const GradSegments& seg, float* grads, float* block_ss);
struct StatsOut { float policy_loss, entropy, value_loss, total_loss, grad_norm, clip_scale; int32_t nonfinite; };
hipError_t rmsprop_update(hipStream_t s, int p_int, float* theta, float* g2, const float* grads,
                          const float* block_ss, int n_ss, const float* hp, const float* loss_partials, int n_loss_blocks,
                          StatsOut* stats_a, StatsOut* stats_b, const WeightMirrors& ws);
hipError_t fill_uniforms(hipStream_t s, uint64_t seed, uint64_t offset, float* out, size_t n);

hipError_t delay_us(hipStream_t s, unsigned us);

// host-side Philox4x32-10 (api uses it for parameter initialisation)
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

}  // namespace paac
