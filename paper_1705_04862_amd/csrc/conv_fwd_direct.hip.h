// Forward pass of the second and third convolution with bf16 operands, one sample at a time from LDS.
//
// The input of a sample (20x20x32, 20x20x16 or 9x9x64 values) fits LDS many times over; as a GEMM its
// im2col rows are gathered from global memory again for every tile.  Here a workgroup keeps the
// sample's input in LDS, position-major with the channels contiguous, so that the MFMA A fragment of
// output position (oy, ox) and k-step (ky, kx, 16 channels) is 16 bytes at base(oy, ox) + a
// compile-time offset.  For the stride-2 layer the image is de-interleaved by the parity of x: the
// positions x = 2 ox + kx of consecutive ox are then neighbours, and the position pitch (channels + 8
// elements) is an odd multiple of 16 bytes, so sixteen lanes read sixteen different bank groups; the row
// pitch keeps that true for the lanes behind the end of an output row.
// The four waves are (32-wide block of output channels) x (share of the k-steps); each keeps its
// weights in registers for all samples, the k-shares are added through LDS (every wave finishes a part
// of the block's rows), and bias + ReLU + bf16 results leave through an LDS image as contiguous 16-byte stores.
#pragma once
#include "gemm_bf16.hip.h"

namespace paac {

template <class G>
__global__ __launch_bounds__(256, 2) void conv_fwd_direct_kernel(const bf16_t* __restrict__ in, const bf16_t* __restrict__ Wt,
                                                                 const float* __restrict__ bias, bf16_t* __restrict__ out, int ns) {
    static_assert((G::ST == 1 || G::ST == 2) && G::CIN % 16 == 0 && G::COUT % 32 == 0 && G::COUT <= 64, "layer shape");
    static_assert(G::ST == 1 || G::W % 2 == 0, "x parity planes");
    constexpr int CIN = G::CIN, COUT = G::COUT, KS = G::KS, ST = G::ST;
    constexpr int PI = CIN + 8, PO = COUT + 8;            // position pitches (elements) of the input and output images
    constexpr int NB = COUT / 32, KW = 4 / NB;            // column blocks; waves sharing the k-steps of one block
    constexpr int CSI = CIN / 16, KSTEPS = KS * KS * CSI, KPW = KSTEPS / KW;
    static_assert(KSTEPS % KW == 0, "equal k-shares");
    constexpr int ROWS = G::HO * G::WO, FRAGS = (ROWS + 31) / 32;
    constexpr int IN_POS = G::H * G::W;
    constexpr int IN_CH = IN_POS * CIN / 8, IN_IT = (IN_CH + 255) / 256;
    constexpr int OUT_CH = ROWS * COUT / 8, OUT_IT = (OUT_CH + 255) / 256;
    // image rows (stride 1) or pairs of image rows with their two x-parity planes each (stride 2) start at a
    // pitch that continues the bank sequence of a fragment from one output row to the next
    constexpr int RP = ST == 1 ? bank_continuing_pitch(G::W * PI, G::WO, PI / 8) : bank_continuing_pitch(2 * G::W * PI, G::WO, PI / 8);
    constexpr int IMG_IN = (ST == 1 ? G::H : G::H / 2) * RP;
    static_assert(ST == 1 || G::H % 2 == 0, "pairs of image rows");
    constexpr int IMG = IMG_IN > ROWS * PO ? IMG_IN : ROWS * PO;      // the output image reuses the input image's LDS
    __shared__ __attribute__((aligned(16))) bf16_t img[IMG];
    typedef KShares<NB, KW, FRAGS> KS_;
    __shared__ __attribute__((aligned(16))) float red[KS_::FLOATS];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, half = lane >> 5;
    const int nb = wave % NB, kg = wave / NB;
    const int co = nb * 32 + m;

    // LDS offset (elements) of input (y, x); additive in (2 oy, 2 ox) + (ky, kx) for the stride-2 layer
    auto ioff = [](int y, int x) { return ST == 2 ? (y >> 1) * RP + (((y & 1) * 2 + (x & 1)) * (G::W / 2) + (x >> 1)) * PI : y * RP + x * PI; };
    // offset of k-step ks = (ky, kx, channel group) relative to a row's base
    auto koff = [&](int ks) {
        const int tap = ks / CSI, cs = ks % CSI, ky = tap / KS, kx = tap % KS;
        return ioff(ky, kx) + cs * 16;
    };

    bf16x8 bfr[KPW];
#pragma unroll
    for (int i = 0; i < KPW; ++i)
        bfr[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Wt + (size_t)co * G::KK + (kg * KPW + i) * 16 + half * 8));
    const float bias_r = bias[co];

    int a_off[FRAGS];
#pragma unroll
    for (int f = 0; f < FRAGS; ++f) {
        const int r = min(f * 32 + m, ROWS - 1);          // rows past the map: a valid position, never stored
        a_off[f] = ioff((r / G::WO) * ST, (r % G::WO) * ST) + half * 8;
    }

    u32x4 pin[IN_IT];
    auto prefetch_in = [&](int smp) __attribute__((always_inline)) {
        const bf16_t* base = in + (size_t)smp * (IN_POS * CIN);
#pragma unroll
        for (int i = 0; i < IN_IT; ++i) pin[i] = *reinterpret_cast<const u32x4*>(base + (size_t)min(tid + i * 256, IN_CH - 1) * 8);
    };
    int s = blockIdx.x;
    if (s >= ns) return;
    prefetch_in(s);

    for (; s < ns; s += gridDim.x) {
#pragma unroll
        for (int i = 0; i < IN_IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < IN_CH) {
                const int pos = ch / (CIN / 8), c8 = ch % (CIN / 8);
                *reinterpret_cast<u32x4*>(img + ioff(pos / G::W, pos % G::W) + c8 * 8) = pin[i];
            }
        }
        __syncthreads();
        prefetch_in(min(s + (int)gridDim.x, ns - 1));     // past the end: the last sample again, not used

        f32x16 acc[FRAGS];
#pragma unroll
        for (int f = 0; f < FRAGS; ++f)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[f][q] = 0.f;
        // the fragments of step i + 1 are read while those of i are multiplied
        u32x4 a_cur[FRAGS], a_nxt[FRAGS];
        const int k0 = koff(kg * KPW);
#pragma unroll
        for (int f = 0; f < FRAGS; ++f) a_cur[f] = *reinterpret_cast<const u32x4*>(img + a_off[f] + k0);
#pragma unroll
        for (int i = 0; i < KPW; ++i) {
            if (i + 1 < KPW) {
                const int kn = koff(kg * KPW + i + 1);
#pragma unroll
                for (int f = 0; f < FRAGS; ++f) a_nxt[f] = *reinterpret_cast<const u32x4*>(img + a_off[f] + kn);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int f = 0; f < FRAGS; ++f)
                acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_cur[f]), bfr[i], acc[f], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int f = 0; f < FRAGS; ++f) a_cur[f] = a_nxt[f];
        }
        with_k_share<KW>(kg, [&](auto KG) __attribute__((always_inline)) { KS_::template give<decltype(KG)::value>(acc, red, nb, lane); });
        __syncthreads();                               // the input image has been read by every wave
        with_k_share<KW>(kg, [&](auto KG) __attribute__((always_inline)) {
            constexpr int kgc = decltype(KG)::value;
            KS_::template take<kgc>(acc, red, nb, lane);
            // lanes m and m ^ 1 hold neighbouring channels of one position: one word per pair
#pragma unroll
            for (int f = 0; f < FRAGS; ++f)
#pragma unroll
                for (int gi = 0; gi < KS_::GPO; ++gi)
#pragma unroll
                    for (int q = 4 * (kgc * KS_::GPO + gi); q < 4 * (kgc * KS_::GPO + gi) + 4; q += 2) {
                        const float v0 = fmaxf(acc[f][q] + bias_r, 0.f), v1 = fmaxf(acc[f][q + 1] + bias_r, 0.f);
                        const float o0 = lane_xor1(v0), o1 = lane_xor1(v1);
                        const bool odd = m & 1;
                        const int r = f * 32 + Mma<32>::row(odd ? q + 1 : q, lane);
                        const unsigned w = odd ? pack2(o1, v1) : pack2(v0, o0);
                        if (r < ROWS) *reinterpret_cast<unsigned*>(img + r * PO + (co & ~1)) = w;
                    }
        });
        __syncthreads();                               // the output image is complete
        bf16_t* dst = out + (size_t)s * (ROWS * COUT);
#pragma unroll
        for (int i = 0; i < OUT_IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < OUT_CH) {
                const int pos = ch / (COUT / 8), c8 = ch % (COUT / 8);
                *reinterpret_cast<u32x4*>(dst + (size_t)ch * 8) = *reinterpret_cast<const u32x4*>(img + pos * PO + c8 * 8);
            }
        }
        __syncthreads();                               // the output image has been read: the next input may overwrite it
    }
}

template <class G>
inline hipError_t launch_conv_fwd_direct(hipStream_t s, const bf16_t* in, const bf16_t* Wt, const float* bias, bf16_t* out, int ns) {
    if (ns <= 0) return hipErrorInvalidValue;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    }
    launch_k((conv_fwd_direct_kernel<G>), dim3(std::min(ns, 2 * cus)), dim3(256), s, in, Wt, bias, out, ns);
    return hipGetLastError();
}

}  // namespace paac
