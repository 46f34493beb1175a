// Dense layers of the PAAC network on the MFMA GEMM core: convolution forward / data gradient /
// weight gradient and the hidden fully connected layer, for the two networks of the paper's
// Experiments section (arch_nips: 16@8x8/4, 32@4x4/2, fc 256; arch_nature: 32@8x8/4, 64@4x4/2,
// 64@3x3/1, fc 512; input 4x84x84, no padding).
#include "gemm_core.hip.h"
#include "gemm_reg16.hip.h"
#include "internal.h"

namespace paac {

typedef ConvGeom<4, 84, 84, 8, 4, 16> NipsC1;
typedef ConvGeom<16, 20, 20, 4, 2, 32> NipsC2;
typedef ConvGeom<4, 84, 84, 8, 4, 32> NatC1;
typedef ConvGeom<32, 20, 20, 4, 2, 64> NatC2;
typedef ConvGeom<64, 9, 9, 3, 1, 64> NatC3;

// tile shapes: BM, BN, BK, waves along m / n / k, MFMA edge, register prefetch stages
typedef Tile<128, 32, 32, 4, 1, 1, 32, 3> T128x32;
typedef Tile<64, 32, 64, 2, 1, 2, 32, 4> T64x32;
typedef Tile<32, 32, 64, 1, 1, 4, 32, 4> T32x32;
typedef Tile<64, 64, 32, 2, 2, 1, 32, 3> T64x64;
typedef Tile<32, 64, 64, 1, 2, 2, 32, 4> T32x64;
// eight wavefronts: the k-steps of a tile are split four ways, so a wave's chain of 64-cycle fp32
// MFMAs is half as long as in the four-wave tile of the same shape, without doubling the number of
// workgroups the dispatcher has to start (the batch-of-32 launches are bound by exactly these two).
// Measured at n_e = 32: first layer 10.3 -> 9.2 us; a 32x64 eight-wave tile for the 64-wide layers
// (half the workgroups of the 32x32 tile) was slower, 8.2 -> 9.7 us, and is not used.
typedef Tile<64, 32, 64, 2, 1, 4, 32, 4> T64x32w8;
// 16-row tiles on the 16x16x4 MFMA for the smallest launches (a batch of 32 states in the second and
// third layer): four times the workgroups of the 32x32 tile, a quarter of the chain of MFMAs per wave
// (n_e = 32: third layer 8.5 -> 6.1 us, second 8.3 -> 7.4 us, arch_nips second layer 5.8 -> 4.4 us; a
// 16x32 tile was between the two)
typedef Tile<16, 16, 64, 1, 1, 4, 16, 4> T16x16;

// wide tiles for the data gradient of a strided layer with all parity classes as columns
typedef Tile<64, 128, 32, 2, 2, 1, 32, 3> T64x128;
typedef Tile<32, 128, 32, 1, 4, 1, 32, 3> T32x128;

// big / middle / small tile per output width for single launches, pbig / pmid / psmall for launches
// that pair two GEMMs (four waves each); wg = tile of the weight-gradient GEMMs.  A 16-wide
// output (first layer of arch_nips) runs on the 32-wide tiles: the upper 16 columns load zeros and
// are not stored (these launches are bound by latency, not by the matrix pipes).
template <int N> struct TileForN;
template <> struct TileForN<16> {
    typedef T128x32 big; typedef T64x32w8 mid; typedef T32x32 small; typedef T64x32 wg;
    typedef T128x32 pbig; typedef T64x32 pmid; typedef T32x32 psmall;
};
template <> struct TileForN<32> {
    typedef T128x32 big; typedef T64x32w8 mid; typedef T32x32 small; typedef T64x32 wg;
    typedef T128x32 pbig; typedef T64x32 pmid; typedef T32x32 psmall;
};
template <> struct TileForN<64> {
    typedef T64x64 big; typedef T32x64 mid; typedef T32x32 small; typedef T64x64 wg;
    typedef T64x64 pbig; typedef T32x64 pmid; typedef T32x32 psmall;
};

// Workgroups are dispatched at a finite rate (on the order of 100 per microsecond), so a launch of
// thousands of small workgroups is bound by dispatch: take the largest tile that still gives about
// one workgroup per compute unit (256 of them).
static const int kMinWgs = 192;
template <class TBig, class TMid, class TSmall, class AL, class BL, class EP>
static hipError_t launch_auto(hipStream_t s, const AL& al, const BL& bl, const EP& ep, int M, int N, int K, int z) {
    auto wgs = [&](int bm, int bn) { return (long)((M + bm - 1) / bm) * ((N + bn - 1) / bn) * z; };
    if (wgs(TBig::BM, TBig::BN) >= kMinWgs) return launch_gemm<TBig>(s, al, bl, ep, M, N, K, z, 0);
    if (wgs(TMid::BM, TMid::BN) >= kMinWgs) return launch_gemm<TMid>(s, al, bl, ep, M, N, K, z, 0);
    if (wgs(TSmall::BM, TSmall::BN) < kMinWgs) {
        if constexpr (std::is_same_v<BL, DenseKCols> && AL::kContig && !SplitAddr<EP>::value && !EP::kColSum)
            return launch_gemm_reg16(s, al, bl, ep, M, N, K, z, 0);
        else
            return launch_gemm<T16x16>(s, al, bl, ep, M, N, K, z, 0);
    }
    return launch_gemm<TSmall>(s, al, bl, ep, M, N, K, z, 0);
}

NetDesc make_net(int arch, int n_actions) {
    NetDesc n{};
    n.arch = arch;
    n.n_actions = n_actions;
    auto set = [](ConvDesc& c, int cin, int h, int w, int ks, int st, int cout) {
        c.cin = cin; c.h = h; c.w = w; c.ks = ks; c.st = st; c.cout = cout;
        c.ho = (h - ks) / st + 1; c.wo = (w - ks) / st + 1; c.kk = ks * ks * cin;
    };
    if (arch == 0) {
        n.n_conv = 2;
        set(n.conv[0], 4, 84, 84, 8, 4, 16);
        set(n.conv[1], 16, 20, 20, 4, 2, 32);
        n.fc = 256;
    } else {
        n.n_conv = 3;
        set(n.conv[0], 4, 84, 84, 8, 4, 32);
        set(n.conv[1], 32, 20, 20, 4, 2, 64);
        set(n.conv[2], 64, 9, 9, 3, 1, 64);
        n.fc = 512;
    }
    const ConvDesc& l = n.conv[n.n_conv - 1];
    n.flat = l.ho * l.wo * l.cout;
    return n;
}

Split plan_split(int k_total, int tiles, int granule, int target_wgs) {
    int n = target_wgs / (tiles > 0 ? tiles : 1);
    if (n < 1) n = 1;
    int k_per = (k_total + n - 1) / n;
    k_per = (k_per + granule - 1) / granule * granule;
    if (k_per < granule) k_per = granule;
    Split s;
    s.k_per = k_per;
    s.n = (k_total + k_per - 1) / k_per;
    if (s.n < 1) s.n = 1;
    return s;
}

// ---------------------------------------------------------------------------------- forward
template <class G>
static hipError_t conv_fwd_f32(hipStream_t s, const void* in, const float* W, const float* b, float* out, int ns) {
    typedef TileForN<G::COUT> TS;
    const int M = ns * G::HO * G::WO;
    ConvNHWCRowsK<G> al{(const float*)in, M};
    DenseKCols bl{W, G::COUT, G::COUT};
    EpiBiasRelu ep{out, b, G::COUT};
    // up to 64 samples the register-only 16x16 kernel also beats the 32x32 tiles that launch_auto would
    // pick from 38 samples on (whole step at n_e = 48: +1.2 %, 64: +1.0 %; at 90 it loses 0.7 %)
    // the third layer (49 rows per sample, 392 tiles of 16x16 at n_e = 32) on 16x32 tiles: 6.0 -> 5.55 us per select
    // call; the second layer on them 6.95 -> 7.2 us (and on 32x16 tiles 6.7 -> 7.9 us), the third on 16x64 8.1 us
    if (ns <= 64 && G::ST == 1) return launch_gemm_reg16<2>(s, al, bl, ep, M, G::COUT, G::KK, 1, 0);
    if (ns <= 64) return launch_gemm_reg16(s, al, bl, ep, M, G::COUT, G::KK, 1, 0);
    return launch_auto<typename TS::big, typename TS::mid, typename TS::small>(s, al, bl, ep, M, G::COUT, G::KK, 1);
}

// layers 1.. of the fp32 path (the first layer runs in conv1_fwd_exact)
hipError_t conv_fwd(hipStream_t s, int arch, int layer, const void* in, const float* W, const float* b,
                    float* out, int ns) {
    if (arch == 0) {
        if (layer == 1) return conv_fwd_f32<NipsC2>(s, in, W, b, out, ns);
    } else {
        if (layer == 1) return conv_fwd_f32<NatC2>(s, in, W, b, out, ns);
        if (layer == 2) return conv_fwd_f32<NatC3>(s, in, W, b, out, ns);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------- data gradient
template <class G>
static hipError_t conv_dgrad_t(hipStream_t s, const float* dy, const float* W, const float* act_in, float* dx, int ns) {
    typedef TileForN<G::CIN> TS;
    const int M = ns * G::HC * G::WC;     // rows per parity class
    DgradGatherRowsK<G> al{dy, M};
    DgradWeightColsK<G> bl{W};
    EpiDgradMask<G> ep{dx, act_in};
    return launch_auto<typename TS::big, typename TS::mid, typename TS::small>(s, al, bl, ep, M, G::CIN, G::KD, G::ST * G::ST);
}

hipError_t conv_dgrad(hipStream_t s, int arch, int layer, const float* dy, const float* W,
                      const float* act_in, float* dx, int ns) {
    if (arch == 0 && layer == 1) return conv_dgrad_t<NipsC2>(s, dy, W, act_in, dx, ns);
    if (arch == 1 && layer == 1) return conv_dgrad_t<NatC2>(s, dy, W, act_in, dx, ns);
    if (arch == 1 && layer == 2) return conv_dgrad_t<NatC3>(s, dy, W, act_in, dx, ns);
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------- weight gradient
template <class G> static int wgrad_tiles_t() {
    typedef typename TileForN<G::COUT>::wg T;
    return ((G::KK + T::BM - 1) / T::BM) * ((G::COUT + T::BN - 1) / T::BN);
}
// layers 1.. (the first layer's weight gradient runs in conv1_wgrad_direct)
int conv_wgrad_tiles(int arch, int layer) {
    if (arch == 0) return wgrad_tiles_t<NipsC2>();
    return layer == 1 ? wgrad_tiles_t<NatC2>() : wgrad_tiles_t<NatC3>();
}

template <class G>
static hipError_t conv_wgrad_t(hipStream_t s, const void* in, const float* dy, float* pw, float* pb, int ns, Split sp) {
    typedef typename TileForN<G::COUT>::wg T;
    const int R = ns * G::HO * G::WO;     // reduction length
    DenseKCols bl{dy, G::COUT, G::COUT};
    EpiPartial<true> ep{pw, (size_t)G::KK * G::COUT, G::COUT, pb, G::COUT};
    ConvNHWCKCols<G> al{(const float*)in, R};
    return launch_gemm<T>(s, al, bl, ep, G::KK, G::COUT, R, sp.n, sp.k_per);
}

hipError_t conv_wgrad(hipStream_t s, int arch, int layer, const void* in, const float* dy, float* pw, float* pb,
                      int ns, Split sp) {
    if (arch == 0) {
        if (layer == 1) return conv_wgrad_t<NipsC2>(s, in, dy, pw, pb, ns, sp);
    } else {
        if (layer == 1) return conv_wgrad_t<NatC2>(s, in, dy, pw, pb, ns, sp);
        if (layer == 2) return conv_wgrad_t<NatC3>(s, in, dy, pw, pb, ns, sp);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------- fused backward of one layer
// The data gradient and the weight gradient of a layer both start from dY and are independent of
// each other: one launch runs both (the chain conv3 -> conv2 of data gradients is the critical path
// of the backward pass, the weight gradients ride along).
template <class TD, class G, class CW>
static hipError_t conv_bwd_pair(hipStream_t s, const float* dy, const float* W, const float* act_in, float* dx, int ns,
                                const CW& wcall) {
    const int M = ns * G::HC * G::WC;
    DgradGatherRowsK<G> al{dy, M};
    DgradWeightColsK<G> bl{W};
    EpiDgradMask<G> ep{dx, act_in};
    return launch_pair(s, make_call<TD>(al, bl, ep, M, G::CIN, G::KD, G::ST * G::ST, 0), wcall);
}

// A strided layer's parity classes share their gathered dY rows: all classes as columns of one GEMM.
template <class TD, class G, class CW>
static hipError_t conv_bwd_pair_all(hipStream_t s, const float* dy, const float* W, const float* act_in, float* dx, int ns,
                                    const CW& wcall) {
    const int M = ns * G::HC * G::WC;
    DgradGatherRowsK<G> al{dy, M};
    DgradWeightColsKAll<G> bl{W};
    EpiDgradMaskAll<G> ep{dx, act_in};
    return launch_pair(s, make_call<TD>(al, bl, ep, M, G::ST * G::ST * G::CIN, G::KD, 1, 0), wcall);
}

template <class G>
static hipError_t conv_bwd_t(hipStream_t s, const float* act_in, const float* dy, const float* W, float* dx, float* pw,
                             float* pb, int ns, Split sp) {
    typedef TileForN<G::CIN> TS;
    const int R = ns * G::HO * G::WO, M = ns * G::HC * G::WC, z = G::ST * G::ST;
    ConvNHWCKCols<G> wal{act_in, R};
    DenseKCols wbl{dy, G::COUT, G::COUT};
    EpiPartial<true> wep{pw, (size_t)G::KK * G::COUT, G::COUT, pb, G::COUT};
    const auto wcall = make_call<typename TileForN<G::COUT>::wg>(wal, wbl, wep, G::KK, G::COUT, R, sp.n, sp.k_per);
    if constexpr (G::ST > 1) {
        constexpr int NA = G::ST * G::ST * G::CIN;
        if constexpr (NA == 128) {
            if ((M + 63) / 64 >= kMinWgs) return conv_bwd_pair_all<T64x128, G>(s, dy, W, act_in, dx, ns, wcall);
            if ((M + 31) / 32 >= kMinWgs) return conv_bwd_pair_all<T32x128, G>(s, dy, W, act_in, dx, ns, wcall);
        } else if constexpr (NA == 64) {
            if ((M + 63) / 64 >= kMinWgs) return conv_bwd_pair_all<T64x64, G>(s, dy, W, act_in, dx, ns, wcall);
            if ((M + 31) / 32 >= kMinWgs) return conv_bwd_pair_all<T32x64, G>(s, dy, W, act_in, dx, ns, wcall);
        }
    }
    auto wgs = [&](int bm, int bn) { return (long)((M + bm - 1) / bm) * ((G::CIN + bn - 1) / bn) * z; };
    if (wgs(TS::pbig::BM, TS::pbig::BN) >= kMinWgs) return conv_bwd_pair<typename TS::pbig, G>(s, dy, W, act_in, dx, ns, wcall);
    if (wgs(TS::pmid::BM, TS::pmid::BN) >= kMinWgs) return conv_bwd_pair<typename TS::pmid, G>(s, dy, W, act_in, dx, ns, wcall);
    return conv_bwd_pair<typename TS::psmall, G>(s, dy, W, act_in, dx, ns, wcall);
}

hipError_t conv_bwd(hipStream_t s, int arch, int layer, const float* act_in, const float* dy, const float* W, float* dx,
                    float* pw, float* pb, int ns, Split sp) {
    if (arch == 0 && layer == 1) return conv_bwd_t<NipsC2>(s, act_in, dy, W, dx, pw, pb, ns, sp);
    if (arch == 1 && layer == 1) return conv_bwd_t<NatC2>(s, act_in, dy, W, dx, pw, pb, ns, sp);
    if (arch == 1 && layer == 2) return conv_bwd_t<NatC3>(s, act_in, dy, W, dx, pw, pb, ns, sp);
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------- fully connected
static void fc_dims(int arch, int& flat, int& fc) {
    if (arch == 0) { flat = 2592; fc = 256; } else { flat = 3136; fc = 512; }
}
static bool fc_small(int ns) { return ns <= 48; }

// up to 48 rows: 16x16 tiles and about 512 workgroups (fewer, longer k-splits than with wider tiles:
// fewer partial sums for the heads kernel to add; arch_nips select: fc 4.5 -> 4.2 us, heads 5.4 -> 4.6 us)
int fc_fwd_target_wgs(int ns) { return fc_small(ns) ? 512 : 256; }
// 49 to 64 rows: 32x32 tiles, four times the tiles of the 64x64 ones and so a quarter of the k-splits, each
// of which is a partial sum for the heads kernel to add (n_e = 64: heads 5.8 -> 4.65 us per select call, the
// GEMM unchanged, step +1.5 %; at 128 rows +0.3 %, at 256 -1.2 %)
static bool fc_mid(int ns) { return ns <= 64; }
int fc_fwd_tiles(int arch, int ns) {
    int flat, fc; fc_dims(arch, flat, fc);
    if (fc_small(ns)) return ((ns + 15) / 16) * (fc / 16);
    if (fc_mid(ns)) return ((ns + 31) / 32) * (fc / 32);
    return ((ns + 63) / 64) * (fc / 64);
}

hipError_t fc_fwd(hipStream_t s, int arch, const float* x, const float* W, float* partial, int ns, Split sp) {
    int flat, fc; fc_dims(arch, flat, fc);
    DenseRowsK al{x, ns, flat};
    DenseKCols bl{W, fc, fc};
    EpiPartial<false> ep{partial, (size_t)ns * fc, fc, nullptr, 0};
    if (fc_small(ns)) return launch_gemm_reg16(s, al, bl, ep, ns, fc, flat, sp.n, sp.k_per);
    if (fc_mid(ns)) return launch_gemm<T32x32>(s, al, bl, ep, ns, fc, flat, sp.n, sp.k_per);
    return launch_gemm<T64x64>(s, al, bl, ep, ns, fc, flat, sp.n, sp.k_per);
}

hipError_t fc_dgrad(hipStream_t s, int arch, const float* dh, const float* W, const float* act, float* dx, int ns) {
    int flat, fc; fc_dims(arch, flat, fc);
    DenseRowsK al{dh, ns, fc};
    DenseRowsK bl{W, flat, fc};          // B(k = j, n = i) = W[i][j]
    EpiDenseMask ep{dx, act, flat};
    return launch_auto<T64x64, T32x64, T32x64>(s, al, bl, ep, ns, flat, fc, 1);
}

int fc_wgrad_tiles(int arch) {
    int flat, fc; fc_dims(arch, flat, fc);
    return ((flat + 63) / 64) * (fc / 64);
}

hipError_t fc_wgrad(hipStream_t s, int arch, const float* x, const float* dh, float* pw, float* pb, int ns, Split sp) {
    int flat, fc; fc_dims(arch, flat, fc);
    DenseKCols al{x, flat, flat};        // A(m = i, k = sample) = x[sample][i]
    DenseKCols bl{dh, fc, fc};
    EpiPartial<true> ep{pw, (size_t)flat * fc, fc, pb, fc};
    return launch_gemm<T64x64>(s, al, bl, ep, flat, fc, ns, sp.n, sp.k_per);
}

// data gradient and weight gradient of the fully connected layer in one launch
hipError_t fc_bwd(hipStream_t s, int arch, const float* x, const float* dh, const float* W, float* dx, float* pw, float* pb,
                  int ns, Split sp) {
    int flat, fc; fc_dims(arch, flat, fc);
    DenseKCols wal{x, flat, flat};
    DenseKCols wbl{dh, fc, fc};
    EpiPartial<true> wep{pw, (size_t)flat * fc, fc, pb, fc};
    // arch_nature, 128 to 384 rows: the weight gradient on 64x128 tiles.  Its reduction dimension is the batch, a
    // handful of k tiles, so a workgroup's start-up and its 16 KB of output stores weigh as much as its
    // MFMAs; the wider tile halves the workgroups and doubles the MFMAs of each (n_e = 32: 21.2 -> 19.05 us,
    // n_e = 64: 35.9 -> 31.5; at 80 rows 13.7 -> 15.2, at 640 rows 55 -> 69, arch_nips at 160 rows 11.7 -> 15.5: not there)
    if (arch == 1 && ns >= 128 && ns <= 384) {
        const auto wide = make_call<T64x128>(wal, wbl, wep, flat, fc, ns, sp.n, sp.k_per);
        DenseRowsK al{dh, ns, fc};
        DenseRowsK bl{W, flat, fc};
        EpiDenseMask ep{dx, x, flat};
        if ((long)((ns + 63) / 64) * (flat / 64) >= kMinWgs) return launch_pair(s, make_call<T64x64>(al, bl, ep, ns, flat, fc, 1, 0), wide);
        return launch_pair(s, make_call<T32x64>(al, bl, ep, ns, flat, fc, 1, 0), wide);
    }
    const auto wcall = make_call<T64x64>(wal, wbl, wep, flat, fc, ns, sp.n, sp.k_per);
    DenseRowsK al{dh, ns, fc};
    DenseRowsK bl{W, flat, fc};
    EpiDenseMask ep{dx, x, flat};
    if ((long)((ns + 63) / 64) * (flat / 64) >= kMinWgs) return launch_pair(s, make_call<T64x64>(al, bl, ep, ns, flat, fc, 1, 0), wcall);
    return launch_pair(s, make_call<T32x64>(al, bl, ep, ns, flat, fc, 1, 0), wcall);
}

}  // namespace paac
