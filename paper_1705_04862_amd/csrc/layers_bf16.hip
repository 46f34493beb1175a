// Dense layers of the PAAC network with bf16 operands (bf16 activations and weight copies, fp32
// accumulation and fp32 gradients): the same six contractions as layers.hip on the bf16 GEMM core.
#include "conv1_direct.hip.h"
#include "conv1_wgrad_direct.hip.h"
#include "conv_dgrad_direct.hip.h"
#include "conv_fwd_direct.hip.h"
#include "conv_fwd_exact.hip.h"
#include "conv_wgrad_direct.hip.h"
#include "internal.h"

namespace paac {

typedef ConvGeom<4, 84, 84, 8, 4, 16> NipsC1;
typedef ConvGeom<16, 20, 20, 4, 2, 32> NipsC2;
typedef ConvGeom<4, 84, 84, 8, 4, 32> NatC1;
typedef ConvGeom<32, 20, 20, 4, 2, 64> NatC2;
typedef ConvGeom<64, 9, 9, 3, 1, 64> NatC3;

// 128 rows, four waves along m; 32 or 64 columns (a 16-wide output uses the 32-wide tile)
typedef TileB<128, 32, 64, 4, 1, 3, 3> B128x32;
typedef TileB<128, 64, 64, 4, 1, 3> B128x64;
typedef TileB<64, 64, 64, 2, 2, 3> B64x64;
// plain fc GEMMs: 2 x 2 fragments per wave, so that two LDS fragment reads feed two MFMAs each
// (the 128x64 tile with four waves along m reads three fragments for two MFMAs and is bound by LDS reads)
typedef TileB<128, 128, 32, 2, 2, 3> B128x128;
// 64-deep k tiles with two register stages: half as many barriers per MFMA (config 4: fc forward 112 -> 100 us,
// fc weight gradient 165 -> 135 us); the data gradient, whose output tile needs registers of its own, spills with it
typedef TileB<128, 128, 64, 2, 2, 2> B128x128K64;
template <int N> struct TileBForN { typedef B128x64 type; };
template <> struct TileBForN<16> { typedef B128x32 type; };
template <> struct TileBForN<32> { typedef B128x32 type; };

// ---------------------------------------------------------------------------------- forward
// first layer: bytes straight from the image; layers 2 and 3: one sample at a time from LDS
hipError_t conv_fwd_bf16(hipStream_t s, int arch, int layer, const void* in, const bf16_t* Wt, const float* b,
                         bf16_t* out, int ns) {
    if (arch == 0) {
        if (layer == 0) return launch_conv1_direct<NipsC1>(s, (const uint8_t*)in, Wt, b, out, ns);
        if (layer == 1) return launch_conv_fwd_direct<NipsC2>(s, (const bf16_t*)in, Wt, b, out, ns);
    } else {
        if (layer == 0) return launch_conv1_direct<NatC1>(s, (const uint8_t*)in, Wt, b, out, ns);
        if (layer == 1) return launch_conv_fwd_direct<NatC2>(s, (const bf16_t*)in, Wt, b, out, ns);
        if (layer == 2) return launch_conv_fwd_direct<NatC3>(s, (const bf16_t*)in, Wt, b, out, ns);
    }
    return hipErrorInvalidValue;
}

// First convolution of the fp32 path: bf16 matrix cores on exact operands (see conv1_exact_kernel).
hipError_t conv1_fwd_exact(hipStream_t s, int arch, const uint8_t* x, const bf16_t* Wk, const float* b, float* out, int ns) {
    if (arch == 0) return launch_conv1_exact<NipsC1>(s, x, Wk, b, out, ns);
    return launch_conv1_exact<NatC1>(s, x, Wk, b, out, ns);
}

// Layers 1.. of the fp32 path on exact bf16 parts, one sample per workgroup (see conv_fwd_exact_kernel).
hipError_t conv_fwd_exact(hipStream_t s, int arch, int layer, const float* in, const bf16_t* Wp, const float* b, float* out, int ns) {
    if (arch == 0 && layer == 1) return launch_conv_fwd_exact<NipsC2>(s, in, Wp, b, out, ns);
    if (arch == 1 && layer == 1) return launch_conv_fwd_exact<NatC2>(s, in, Wp, b, out, ns);
    if (arch == 1 && layer == 2) return launch_conv_fwd_exact<NatC3>(s, in, Wp, b, out, ns);
    return hipErrorInvalidValue;
}

// All convolutions of the fp32 path in one launch, one workgroup per sample (see trunk_fwd_exact_kernel);
// w[l], b[l], out[l]: weight parts, bias and fp32 NHWC output of layer l.  ns <= trunk_fwd_exact_max().
int trunk_fwd_exact_max() { return device_cus(); }
hipError_t trunk_fwd_exact(hipStream_t s, int arch, const uint8_t* x, const bf16_t* const* w, const float* const* b, float* const* out, int ns) {
    if (arch == 0) return launch_trunk_fwd_exact<NipsC1, NipsC2, NoLayer>(s, x, w[0], b[0], out[0], w[1], b[1], out[1], nullptr, nullptr, nullptr, ns);
    return launch_trunk_fwd_exact<NatC1, NatC2, NatC3>(s, x, w[0], b[0], out[0], w[1], b[1], out[1], w[2], b[2], out[2], ns);
}

// First convolution's weight gradient straight from the image (see conv1_wgrad_direct_kernel): dy is
// fp32 when exact (fp32 path) and bf16 otherwise; n_wgs partials are written.
hipError_t conv1_wgrad_direct(hipStream_t s, int arch, bool exact, const uint8_t* x, const void* dy, float* pw, float* pb, int ns, int n_wgs) {
    if (arch == 0) return exact ? launch_conv1_wgrad_direct<NipsC1, true>(s, x, dy, pw, pb, ns, n_wgs)
                                : launch_conv1_wgrad_direct<NipsC1, false>(s, x, dy, pw, pb, ns, n_wgs);
    return exact ? launch_conv1_wgrad_direct<NatC1, true>(s, x, dy, pw, pb, ns, n_wgs)
                 : launch_conv1_wgrad_direct<NatC1, false>(s, x, dy, pw, pb, ns, n_wgs);
}

// ---------------------------------------------------------------------------------- data gradient
hipError_t conv_dgrad_bf16(hipStream_t s, int arch, int layer, const bf16_t* dy, const bf16_t* Wd, const bf16_t* act_in,
                           bf16_t* dx, int ns) {
    // one sample at a time from LDS
    if (arch == 0 && layer == 1) return launch_conv_dgrad_direct<NipsC2>(s, dy, Wd, act_in, dx, ns);
    if (arch == 1 && layer == 1) return launch_conv_dgrad_direct<NatC2>(s, dy, Wd, act_in, dx, ns);
    if (arch == 1 && layer == 2) return launch_conv_dgrad_direct_s1<NatC3>(s, dy, Wd, act_in, dx, ns);
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------- weight gradient
template <class G> static int wgrad_tiles_t() {
    typedef typename TileBForN<G::COUT>::type T;
    return ((G::KK + T::BM - 1) / T::BM) * ((G::COUT + T::BN - 1) / T::BN);
}
// layers 1.. (the first layer's weight gradient runs in conv1_wgrad_direct)
int conv_wgrad_tiles_bf16(int arch, int layer) {
    if (arch == 0) return wgrad_tiles_t<NipsC2>();
    return layer == 1 ? wgrad_tiles_t<NatC2>() : wgrad_tiles_t<NatC3>();
}

template <class G>
static hipError_t conv_wgrad_t(hipStream_t s, const void* in, const bf16_t* dy, float* pw, float* pb, int ns, Split sp) {
    typedef typename TileBForN<G::COUT>::type T;
    const int R = ns * G::HO * G::WO;
    DenseKCols8 bl{dy, G::COUT, G::COUT};
    EpiPartial<true> ep{pw, (size_t)G::KK * G::COUT, G::COUT, pb, G::COUT};
    ConvNHWCKCols8<G> al{(const bf16_t*)in, R};
    return launch_gemm_bf16<T>(s, al, bl, ep, G::KK, G::COUT, R, sp.n, sp.k_per);
}

// Workgroups (= partial sums) of the per-sample weight-gradient kernel, 0 where the tiled GEMM is used.
// From 2048 samples on: below, a workgroup has too few samples to pay for one partial sum per
// compute unit (256 partial sums per tensor for the reduction to add), and the GEMMs are as fast.
int conv_wgrad_direct_wgs(int arch, int layer, int ns) {
    if (arch != 1 || layer < 1 || ns < 2048) return 0;
    return std::min(ns, device_cus());
}

hipError_t conv_wgrad_bf16(hipStream_t s, int arch, int layer, const void* in, const bf16_t* dy, float* pw, float* pb,
                           int ns, Split sp) {
    if (arch == 1 && sp.k_per == 0) {                  // one sample at a time from LDS, sp.n workgroups
        if (layer == 1) return launch_conv_wgrad_direct<NatC2>(s, (const bf16_t*)in, dy, pw, pb, ns, sp.n);
        if (layer == 2) return launch_conv_wgrad_direct<NatC3>(s, (const bf16_t*)in, dy, pw, pb, ns, sp.n);
    }
    if (arch == 0) {
        if (layer == 1) return conv_wgrad_t<NipsC2>(s, in, dy, pw, pb, ns, sp);
    } else {
        if (layer == 1) return conv_wgrad_t<NatC2>(s, in, dy, pw, pb, ns, sp);
        if (layer == 2) return conv_wgrad_t<NatC3>(s, in, dy, pw, pb, ns, sp);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------- fully connected
static void fc_dims(int arch, int& flat, int& fc) {
    if (arch == 0) { flat = 2592; fc = 256; } else { flat = 3136; fc = 512; }
}

// up to 1024 rows (select calls) the narrower tile gives more workgroups and is faster
static bool fc_fwd_wide(int ns) { return ns > 1024; }
// up to 256 rows 64-row tiles: twice the tiles, so half as many k-splits fill the chip, and every split is a
// partial sum that the heads kernel has to add (n_e = 256: fc 7.7 -> 6.2 us, heads 6.2 -> 5.4 us per select
// call; n_e = 128: 7.4 -> 5.4 and 6.1 -> 5.3; at 512 rows the step did not gain)
static bool fc_fwd_64(int ns) { return ns <= 256; }
int fc_fwd_tiles_bf16(int arch, int ns) {
    int flat, fc; fc_dims(arch, flat, fc);
    if (fc_fwd_64(ns)) return ((ns + 63) / 64) * (fc / 64);
    return ((ns + 127) / 128) * (fc / (fc_fwd_wide(ns) ? 128 : 64));
}

// partial[split][ns][fc] (fp32) = x[ns][flat] . Wt[fc][flat]^T
hipError_t fc_fwd_bf16(hipStream_t s, int arch, const bf16_t* x, const bf16_t* Wt, float* partial, int ns, Split sp) {
    int flat, fc; fc_dims(arch, flat, fc);
    DenseRowsK8 al{x, ns, flat};
    DenseRowsK8 bl{Wt, fc, flat};
    EpiPartial<false> ep{partial, (size_t)ns * fc, fc, nullptr, 0};
    if (fc_fwd_wide(ns)) return launch_gemm_bf16<B128x128K64>(s, al, bl, ep, ns, fc, flat, sp.n, sp.k_per, 1);
    if (fc_fwd_64(ns)) return launch_gemm_bf16<B64x64>(s, al, bl, ep, ns, fc, flat, sp.n, sp.k_per, 1);
    return launch_gemm_bf16<B128x64>(s, al, bl, ep, ns, fc, flat, sp.n, sp.k_per, 1);
}

// dx[ns][flat] = (dh[ns][fc] . W[flat][fc]^T) * 1[act > 0]
hipError_t fc_dgrad_bf16(hipStream_t s, int arch, const bf16_t* dh, const bf16_t* Wc, const bf16_t* act, bf16_t* dx, int ns) {
    int flat, fc; fc_dims(arch, flat, fc);
    DenseRowsK8 al{dh, ns, fc};
    DenseRowsK8 bl{Wc, flat, fc};
    EpiDenseMaskB ep{dx, act, flat, nullptr};
    // a small batch gives too few of the wide tiles
    if (ns >= 4096) return launch_gemm_bf16<B128x128>(s, al, bl, ep, ns, flat, fc, 1, 0);
    return launch_gemm_bf16<B128x64>(s, al, bl, ep, ns, flat, fc, 1, 0);
}

int fc_wgrad_tiles_bf16(int arch) {
    int flat, fc; fc_dims(arch, flat, fc);
    return ((flat + 127) / 128) * (fc / 128);
}

hipError_t fc_wgrad_bf16(hipStream_t s, int arch, const bf16_t* x, const bf16_t* dh, float* pw, float* pb, int ns, Split sp) {
    int flat, fc; fc_dims(arch, flat, fc);
    DenseKCols8 al{x, flat, flat};
    DenseKCols8 bl{dh, fc, fc};
    EpiPartial<true> ep{pw, (size_t)flat * fc, fc, pb, fc};
    return launch_gemm_bf16<B128x128K64>(s, al, bl, ep, flat, fc, ns, sp.n, sp.k_per, 1);
}

// ---------------------------------------------------------------------------------- bf16 weight copies
// One launch rewrites every bf16 copy from the fp32 master arena:
//   mode 0: dst[c*K + k]              = src[k*C + c]           (forward: [c_out][K])
//   mode 1: dst[i]                    = src[i]                 (fc data gradient: [flat][fc])
//   mode 2: dst[(ci*T + t)*C + co]    = src[(t*CIN + ci)*C + co]   (conv data gradient: [ci][ky,kx][co])
//   mode 3: dst[(k/8)*256 + c*8 + k%8] = src[k*C + c], zero for c in [C, 32)   (first layer forward: the
//           order in which the lanes read their MFMA B fragments, one contiguous KB per wave and load)
__global__ __launch_bounds__(256) void make_bf16_weights_kernel(const WeightCopies w, const float* theta) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= w.total) return;
    int sidx = 0;
    for (int q = 1; q < w.n; ++q) if (i >= w.start[q]) sidx = q;
    const int o = i - w.start[sidx];
    const int K = w.K[sidx], C = w.C[sidx];
    const float* src = theta + w.src_off[sidx];
    int si;
    if (w.mode[sidx] == 0) { const int c = o / K, k = o % K; si = k * C + c; }
    else if (w.mode[sidx] == 1) si = o;
    else if (w.mode[sidx] == 3) {
        const int c = (o % 256) / 8, k = (o / 256) * 8 + o % 8;
        if (c >= C) { w.dst[sidx][o] = 0; return; }
        si = k * C + c;
    } else {
        const int T = K / w.cin[sidx];                      // taps
        const int co = o % C, t = (o / C) % T, ci = o / (C * T);
        si = (t * w.cin[sidx] + ci) * C + co;
    }
    w.dst[sidx][o] = f2bf(src[si]);
}

hipError_t make_bf16_weights(hipStream_t s, const WeightCopies& w, const float* theta) {
    launch_k(make_bf16_weights_kernel, dim3((w.total + 255) / 256), dim3(256), s, w, theta);
    return hipGetLastError();
}

}  // namespace paac
