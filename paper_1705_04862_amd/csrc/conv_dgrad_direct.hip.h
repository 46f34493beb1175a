// Data gradient of a stride-2, 4x4 convolution (the second layer of both networks) with bf16
// operands, one sample at a time from LDS.
//
//   dX[y][x][ci] = 1[act_in > 0] * sum over (ky, kx, co) of dY[(y - ky) / 2][(x - kx) / 2][co] W[ky][kx][ci][co]
//
// Input positions fall into 2 x 2 parity classes (py, px) = (y mod 2, x mod 2); the block position
// (yy, xx) = (y / 2, x / 2) of a class sees the 2 x 2 taps dY[yy - ty][xx - tx] with ky = py + 2 ty,
// kx = px + 2 tx.  The GEMM form of this gathers every dY row from global memory per tile and
// scatters 2-byte results; at 81 x C_out values per sample the whole dY of a sample fits LDS many
// times over.  Here a workgroup keeps one sample's dY in LDS with a border of zero positions (the
// taps that fall outside the output map read zeros, no bounds logic at all), wave z owns parity
// class z with its 256 x C_in weights in registers, an MFMA A fragment is 32 block positions read at
// base + compile-time tap offset, and the four classes meet again in an LDS image of the sample's
// dX, which leaves as contiguous 16-byte stores after the ReLU mask (also read as 16-byte loads).
#pragma once
#include "gemm_bf16.hip.h"

namespace paac {

template <class G>
__global__ __launch_bounds__(256, 2) void conv_dgrad_direct_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ Wd,
                                                                   const bf16_t* __restrict__ act_in, bf16_t* __restrict__ dx, int ns) {
    static_assert(G::ST == 2 && G::KS == 4 && G::TAPS == 2 && G::HC * G::ST == G::H && G::WC * G::ST == G::W, "stride-2 4x4 layer");
    static_assert(G::CIN <= 32 && G::CIN % 8 == 0 && G::COUT % 16 == 0, "one 32-wide MFMA column block");
    constexpr int COUT = G::COUT, CIN = G::CIN;
    constexpr int PP = COUT + 8;                       // position pitch of the padded dY (odd multiple of 16 bytes: no bank conflicts)
    constexpr int PADW = G::WO + 2, PADH = G::HO + 2;  // one zero position around the output map
    constexpr int RP = bank_continuing_pitch(PADW * PP, G::WC, PP / 8);     // row pitch: a fragment's bank sequence continues in the next row
    constexpr int OP = CIN + 8;                        // position pitch of the dX image
    constexpr int CS = COUT / 16, KSTEPS = 4 * CS;     // 16-wide k-steps per tap, in all
    constexpr int ROWS = G::HC * G::WC, FRAGS = (ROWS + 31) / 32;
    constexpr int DY_CH = G::HO * G::WO * COUT / 8, DY_IT = (DY_CH + 255) / 256;
    constexpr int DX_CH = G::H * G::W * CIN / 8, DX_IT = (DX_CH + 255) / 256;
    __shared__ __attribute__((aligned(16))) bf16_t dyp[PADH * RP];
    __shared__ __attribute__((aligned(16))) bf16_t dxi[G::H * G::W * OP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, half = lane >> 5;
    const int py = wave >> 1, px = wave & 1;           // this wave's parity class

    // weights of input channel m for this class: B(k = (ty, tx, co), n = ci) = Wd[ci][ky][kx][co]
    bf16x8 bfr[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
        const int tap = ks / CS, cs = ks % CS, ty = tap >> 1, tx = tap & 1;
        const int ky = py + 2 * ty, kx = px + 2 * tx;
        uint4 w = zero_u4();
        if (m < CIN) w = *reinterpret_cast<const uint4*>(Wd + ((size_t)(m * 16 + ky * 4 + kx) * COUT + cs * 16 + half * 8));
        bfr[ks] = __builtin_bit_cast(bf16x8, w);
    }

    // raw data of a sample in registers: dY one sample ahead of the MFMAs, the mask during the epilogue
    u32x4 pdy[DY_IT], pact[DX_IT];
#define PAAC_PREFETCH_DY(S_)                                                                                             \
    {                                                                                                                    \
        const bf16_t* base_ = dy + (size_t)(S_) * (G::HO * G::WO * COUT);                                                \
        _Pragma("unroll") for (int i = 0; i < DY_IT; ++i)                                                                \
            pdy[i] = *reinterpret_cast<const u32x4*>(base_ + (size_t)min(tid + i * 256, DY_CH - 1) * 8);                 \
    }
    int s = blockIdx.x;
    if (s >= ns) return;
    PAAC_PREFETCH_DY(s);
    for (int i = tid; i < PADH * RP / 8; i += 256) reinterpret_cast<uint4*>(dyp)[i] = zero_u4();     // the border stays zero
    __syncthreads();

    // block position of fragment row m (rows past the class: a valid position, never stored)
    int a_off[FRAGS];
#pragma unroll
    for (int f = 0; f < FRAGS; ++f) {
        const int r = min(f * 32 + m, ROWS - 1);
        a_off[f] = (r / G::WC + 1) * RP + (r % G::WC + 1) * PP + half * 8;
    }

    for (; s < ns; s += gridDim.x) {
#pragma unroll
        for (int i = 0; i < DY_IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < DY_CH) {
                const int pos = ch / (COUT / 8), c8 = ch % (COUT / 8);
                *reinterpret_cast<u32x4*>(dyp + (pos / G::WO + 1) * RP + (pos % G::WO + 1) * PP + c8 * 8) = pdy[i];
            }
        }
        __syncthreads();                               // also: the previous sample's dX image has been read
        if (s + (int)gridDim.x < ns) PAAC_PREFETCH_DY(s + gridDim.x);

        f32x16 acc[FRAGS];
#pragma unroll
        for (int f = 0; f < FRAGS; ++f)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[f][q] = 0.f;
        // the fragments of k-step ks + 1 are read while those of ks are multiplied (the scheduling barriers
        // keep the reads ahead: read-wait-multiply in a row would expose the LDS latency 64 times a sample)
        auto koff = [](int ks) { return (ks % CS) * 16 - (((ks / CS) >> 1) * RP + ((ks / CS) & 1) * PP); };   // constant after unrolling
        u32x4 a_cur[FRAGS], a_nxt[FRAGS];
#pragma unroll
        for (int f = 0; f < FRAGS; ++f) a_cur[f] = *reinterpret_cast<const u32x4*>(dyp + a_off[f] + koff(0));
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            if (ks + 1 < KSTEPS) {
#pragma unroll
                for (int f = 0; f < FRAGS; ++f) a_nxt[f] = *reinterpret_cast<const u32x4*>(dyp + a_off[f] + koff(ks + 1));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int f = 0; f < FRAGS; ++f)
                acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_cur[f]), bfr[ks], acc[f], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int f = 0; f < FRAGS; ++f) a_cur[f] = a_nxt[f];
        }
        {                                              // the mask: in flight while the accumulators go to the dX image
            // (requested before the MFMA phase it competes with the next sample's dY for the memory
            // pipe of a kernel that is bound by HBM: measured 6 % slower)
            const bf16_t* base = act_in + (size_t)s * (G::H * G::W * CIN);
#pragma unroll
            for (int i = 0; i < DX_IT; ++i) pact[i] = *reinterpret_cast<const u32x4*>(base + (size_t)min(tid + i * 256, DX_CH - 1) * 8);
        }
        // lanes m and m ^ 1 hold neighbouring channels of the same position: the even lane stores both as
        // one word for even q, the odd lane for odd q (half as many LDS stores, none narrower than a bank word)
#pragma unroll
        for (int f = 0; f < FRAGS; ++f)
#pragma unroll
            for (int q = 0; q < 16; q += 2) {
                const float o0 = lane_xor1(acc[f][q]), o1 = lane_xor1(acc[f][q + 1]);
                const bool odd = m & 1;
                const int r = f * 32 + Mma<32>::row(odd ? q + 1 : q, lane);
                const unsigned w = odd ? pack2(o1, acc[f][q + 1]) : pack2(acc[f][q], o0);
                if (r < ROWS && m < CIN)
                    *reinterpret_cast<unsigned*>(dxi + ((2 * (r / G::WC) + py) * G::W + 2 * (r % G::WC) + px) * OP + (m & ~1)) = w;
            }
        __syncthreads();                               // dY has been read by every wave, the dX image is complete
        bf16_t* out = dx + (size_t)s * (G::H * G::W * CIN);
#pragma unroll
        for (int i = 0; i < DX_IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < DX_CH) {
                const int pos = ch / (CIN / 8), c8 = ch % (CIN / 8);
                uint4 v = *reinterpret_cast<const uint4*>(dxi + pos * OP + c8 * 8);
                v.x = mask2(v.x, pact[i].x); v.y = mask2(v.y, pact[i].y); v.z = mask2(v.z, pact[i].z); v.w = mask2(v.w, pact[i].w);
                *reinterpret_cast<uint4*>(out + (size_t)ch * 8) = v;
            }
        }
    }
}

#undef PAAC_PREFETCH_DY

template <class G>
inline hipError_t launch_conv_dgrad_direct(hipStream_t s, const bf16_t* dy, const bf16_t* Wd, const bf16_t* act_in, bf16_t* dx, int ns) {
    if (ns <= 0) return hipErrorInvalidValue;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    }
    launch_k((conv_dgrad_direct_kernel<G>), dim3(std::min(ns, 2 * cus)), dim3(256), s, dy, Wd, act_in, dx, ns);
    return hipGetLastError();
}

// The stride-1, 3x3 third layer in the same way: dX[y][x][ci] = 1[act_in > 0] * sum over (ky, kx, co)
// of dY[y - ky][x - kx][co] W[ky][kx][ci][co], a full correlation, so the zero border is two positions
// wide.  There are no parity classes; the four waves are 2 halves of the 64 input channels x 2 halves of
// the 36 k-steps (each wave keeps 18 k-steps of weights in registers), and the two k-halves are added
// through LDS (each wave finishes half of its block's rows) before the image of dX is written.
template <class G>
__global__ __launch_bounds__(256, 2) void conv_dgrad_direct_s1_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ Wd,
                                                                      const bf16_t* __restrict__ act_in, bf16_t* __restrict__ dx, int ns) {
    static_assert(G::ST == 1 && G::KS == 3 && G::CIN == 64 && G::COUT % 16 == 0, "stride-1 3x3 layer with 64 input channels");
    constexpr int COUT = G::COUT, CIN = G::CIN, T = G::KS * G::KS;
    constexpr int PP = COUT + 8, PAD = G::KS - 1, PADW = G::WO + 2 * PAD, PADH = G::HO + 2 * PAD;
    constexpr int RP = bank_continuing_pitch(PADW * PP, G::W, PP / 8);      // row pitch: a fragment's bank sequence continues in the next row
    constexpr int OP = CIN + 8;
    constexpr int CS = COUT / 16, KSTEPS = T * CS, KH = KSTEPS / 2;
    static_assert(KSTEPS % 2 == 0, "two equal k-halves");
    constexpr int ROWS = G::H * G::W, FRAGS = (ROWS + 31) / 32;
    constexpr int DY_CH = G::HO * G::WO * COUT / 8, DY_IT = (DY_CH + 255) / 256;
    constexpr int DX_CH = ROWS * CIN / 8, DX_IT = (DX_CH + 255) / 256;
    __shared__ __attribute__((aligned(16))) bf16_t dyp[PADH * RP];
    __shared__ __attribute__((aligned(16))) bf16_t dxi[ROWS * OP];
    typedef KShares<2, 2, FRAGS> KS_;
    __shared__ __attribute__((aligned(16))) float red[KS_::FLOATS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, half = lane >> 5;
    const int nb = wave & 1, kh = wave >> 1;           // half of the input channels, half of the k-steps
    const int ci = nb * 32 + m;

    bf16x8 bfr[KH];
#pragma unroll
    for (int i = 0; i < KH; ++i) {
        // both k-halves are unrolled with compile-time tap offsets below; the weights follow the same ks
        const int ks0 = i, ks1 = KH + i;
        const int t0 = ks0 / CS, c0 = ks0 % CS, t1 = ks1 / CS, c1 = ks1 % CS;
        const uint4 w0 = *reinterpret_cast<const uint4*>(Wd + ((size_t)(ci * T + t0) * COUT + c0 * 16 + half * 8));
        const uint4 w1 = *reinterpret_cast<const uint4*>(Wd + ((size_t)(ci * T + t1) * COUT + c1 * 16 + half * 8));
        bfr[i] = __builtin_bit_cast(bf16x8, kh ? w1 : w0);
    }

    u32x4 pdy[DY_IT], pact[DX_IT];
#define PAAC_PREFETCH_DY(S_)                                                                                             \
    {                                                                                                                    \
        const bf16_t* base_ = dy + (size_t)(S_) * (G::HO * G::WO * COUT);                                                \
        _Pragma("unroll") for (int i = 0; i < DY_IT; ++i)                                                                \
            pdy[i] = *reinterpret_cast<const u32x4*>(base_ + (size_t)min(tid + i * 256, DY_CH - 1) * 8);                 \
    }
    int s = blockIdx.x;
    if (s >= ns) return;
    PAAC_PREFETCH_DY(s);
    for (int i = tid; i < PADH * RP / 8; i += 256) reinterpret_cast<uint4*>(dyp)[i] = zero_u4();     // the border stays zero
    __syncthreads();

    int a_off[FRAGS];
#pragma unroll
    for (int f = 0; f < FRAGS; ++f) {
        const int r = min(f * 32 + m, ROWS - 1);
        a_off[f] = (r / G::W + PAD) * RP + (r % G::W + PAD) * PP + half * 8;
    }

    for (; s < ns; s += gridDim.x) {
#pragma unroll
        for (int i = 0; i < DY_IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < DY_CH) {
                const int pos = ch / (COUT / 8), c8 = ch % (COUT / 8);
                *reinterpret_cast<u32x4*>(dyp + (pos / G::WO + PAD) * RP + (pos % G::WO + PAD) * PP + c8 * 8) = pdy[i];
            }
        }
        __syncthreads();                               // also: the previous sample's dX image has been read
        if (s + (int)gridDim.x < ns) PAAC_PREFETCH_DY(s + gridDim.x);
        {                                              // the mask of this sample: in flight during the whole MFMA phase
            const bf16_t* base = act_in + (size_t)s * (ROWS * CIN);
#pragma unroll
            for (int i = 0; i < DX_IT; ++i) pact[i] = *reinterpret_cast<const u32x4*>(base + (size_t)min(tid + i * 256, DX_CH - 1) * 8);
        }

        f32x16 acc[FRAGS];
#pragma unroll
        for (int f = 0; f < FRAGS; ++f)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[f][q] = 0.f;
        // tap offset of k-step i in either half: a constant per branch, selected by the wave-uniform kh;
        // the fragments of step i + 1 are read while those of i are multiplied
        auto koff = [&](int i) {
            const int ks0 = i, ks1 = KH + i;
            const int off0 = (ks0 % CS) * 16 - ((ks0 / CS / G::KS) * RP + (ks0 / CS % G::KS) * PP);
            const int off1 = (ks1 % CS) * 16 - ((ks1 / CS / G::KS) * RP + (ks1 / CS % G::KS) * PP);
            return kh ? off1 : off0;
        };
        u32x4 a_cur[FRAGS], a_nxt[FRAGS];
#pragma unroll
        for (int f = 0; f < FRAGS; ++f) a_cur[f] = *reinterpret_cast<const u32x4*>(dyp + a_off[f] + koff(0));
#pragma unroll
        for (int i = 0; i < KH; ++i) {
            if (i + 1 < KH) {
#pragma unroll
                for (int f = 0; f < FRAGS; ++f) a_nxt[f] = *reinterpret_cast<const u32x4*>(dyp + a_off[f] + koff(i + 1));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int f = 0; f < FRAGS; ++f)
                acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_cur[f]), bfr[i], acc[f], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int f = 0; f < FRAGS; ++f) a_cur[f] = a_nxt[f];
        }
        with_k_share<2>(kh, [&](auto KG) __attribute__((always_inline)) { KS_::template give<decltype(KG)::value>(acc, red, nb, lane); });
        __syncthreads();                               // dY has been read by every wave
        with_k_share<2>(kh, [&](auto KG) __attribute__((always_inline)) {
            constexpr int kgc = decltype(KG)::value;
            KS_::template take<kgc>(acc, red, nb, lane);
            // lanes m and m ^ 1 hold neighbouring channels of one position: one word per pair
#pragma unroll
            for (int f = 0; f < FRAGS; ++f)
#pragma unroll
                for (int gi = 0; gi < KS_::GPO; ++gi)
#pragma unroll
                    for (int q = 4 * (kgc * KS_::GPO + gi); q < 4 * (kgc * KS_::GPO + gi) + 4; q += 2) {
                        const float o0 = lane_xor1(acc[f][q]), o1 = lane_xor1(acc[f][q + 1]);
                        const bool odd = m & 1;
                        const int r = f * 32 + Mma<32>::row(odd ? q + 1 : q, lane);
                        const unsigned w = odd ? pack2(o1, acc[f][q + 1]) : pack2(acc[f][q], o0);
                        if (r < ROWS) *reinterpret_cast<unsigned*>(dxi + r * OP + (ci & ~1)) = w;
                    }
        });
        __syncthreads();                               // the dX image is complete
        bf16_t* out = dx + (size_t)s * (ROWS * CIN);
#pragma unroll
        for (int i = 0; i < DX_IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < DX_CH) {
                const int pos = ch / (CIN / 8), c8 = ch % (CIN / 8);
                uint4 v = *reinterpret_cast<const uint4*>(dxi + pos * OP + c8 * 8);
                v.x = mask2(v.x, pact[i].x); v.y = mask2(v.y, pact[i].y); v.z = mask2(v.z, pact[i].z); v.w = mask2(v.w, pact[i].w);
                *reinterpret_cast<uint4*>(out + (size_t)ch * 8) = v;
            }
        }
    }
#undef PAAC_PREFETCH_DY
}

template <class G>
inline hipError_t launch_conv_dgrad_direct_s1(hipStream_t s, const bf16_t* dy, const bf16_t* Wd, const bf16_t* act_in, bf16_t* dx, int ns) {
    if (ns <= 0) return hipErrorInvalidValue;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    }
    launch_k((conv_dgrad_direct_s1_kernel<G>), dim3(std::min(ns, 2 * cus)), dim3(256), s, dy, Wd, act_in, dx, ns);
    return hipGetLastError();
}

}  // namespace paac
