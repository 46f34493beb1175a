// Forward pass of the second and third convolution of the fp32 path, one sample at a time from LDS,
// on the bf16 matrix cores with exact operands.
//
// An fp32 number is the sum of three bf16 numbers (its 24 significand bits cut 8 + 8 + 8 by
// truncation); the product of two bf16 numbers is exact in fp32.  a*w = sum over the nine part
// products; the six of order >= 2^-16 are accumulated (the three left out are of relative size
// 2^-24 and below, the rounding level of an fp32 product), each one MFMA of four times the depth and
// twice the rate of the fp32 instruction.  The weights arrive already split, in the order in which
// the lanes read their B fragments (WeightSplits); the activations are split once, when the sample is
// written into LDS as three images.
//
// Layout and wave roles are those of the bf16 kernel (conv_fwd_direct_kernel): position-major images
// with the channels contiguous, de-interleaved by the parity of x for the stride-2 layer, pitch an odd
// multiple of 16 bytes; waves = (32-wide block of output channels) x (share of the k-steps), weights
// in registers, k-shares added through LDS, bias + ReLU results leave through an fp32 LDS image as
// contiguous 16-byte stores.  The grid is one workgroup per sample up to one per compute unit.
#pragma once
#include "gemm_bf16.hip.h"

namespace paac {

// two fp32 numbers -> their three bf16 parts, packed (a in the low half)
__device__ __forceinline__ void split3_pair(float a, float b, unsigned& hi, unsigned& mid, unsigned& lo) {
    const unsigned ah = __float_as_uint(a) & 0xffff0000u, bh = __float_as_uint(b) & 0xffff0000u;
    const float a1 = a - __uint_as_float(ah), b1 = b - __uint_as_float(bh);
    const unsigned am = __float_as_uint(a1) & 0xffff0000u, bm = __float_as_uint(b1) & 0xffff0000u;
    const float a2 = a1 - __uint_as_float(am), b2 = b1 - __uint_as_float(bm);
    hi = (ah >> 16) | bh;
    mid = (am >> 16) | bm;
    lo = __builtin_amdgcn_perm(__float_as_uint(b2), __float_as_uint(a2), 0x07060302u);
}

template <class G> struct ConvFwdExactShape {
    static constexpr int CIN = G::CIN, COUT = G::COUT, KS = G::KS, ST = G::ST;
    static constexpr int PI = CIN + 8, PO = COUT + 8;         // position pitches: bf16 input images, fp32 output image
    static constexpr int NB = COUT / 32, KW = 4 / NB;
    static constexpr int CSI = CIN / 16, KSTEPS = KS * KS * CSI, KPW = KSTEPS / KW;
    static constexpr int ROWS = G::HO * G::WO, FRAGS = (ROWS + 31) / 32;
    static constexpr int IN_POS = G::H * G::W, PLANE = IN_POS * PI;
    static constexpr int IMG_BYTES = (3 * PLANE * 2 > ROWS * PO * 4 ? 3 * PLANE * 2 : ROWS * PO * 4);
    static constexpr int RED_FLOATS = (KW - 1) * NB * FRAGS * 16 * 64;
    static constexpr int LDS_BYTES = IMG_BYTES + RED_FLOATS * 4;
    static_assert(IMG_BYTES % 16 == 0 && (PLANE * 2) % 16 == 0, "16-byte aligned images");
    static_assert(LDS_BYTES <= 160 * 1024, "fits the LDS of a compute unit");
};

template <class G>
__global__ __launch_bounds__(256, 1) void conv_fwd_exact_kernel(const float* __restrict__ in, const bf16_t* __restrict__ Wp,
                                                                const float* __restrict__ bias, float* __restrict__ out, int ns) {
    typedef ConvFwdExactShape<G> S;
    static_assert((G::ST == 1 || G::ST == 2) && G::CIN % 16 == 0 && G::COUT % 32 == 0 && G::COUT <= 64, "layer shape");
    static_assert(G::ST == 1 || G::W % 2 == 0, "x parity planes");
    constexpr int CIN = S::CIN, COUT = S::COUT, KS = S::KS, ST = S::ST, PI = S::PI, PO = S::PO;
    constexpr int NB = S::NB, KW = S::KW, CSI = S::CSI, KSTEPS = S::KSTEPS, KPW = S::KPW;
    static_assert(KSTEPS % KW == 0, "equal k-shares");
    constexpr int ROWS = S::ROWS, FRAGS = S::FRAGS, IN_POS = S::IN_POS, PLANE = S::PLANE;
    constexpr int WPLANE = NB * 32 * G::KK;                   // elements of one part of the weights
    constexpr int IN_CH = IN_POS * CIN / 4, IN_IT = (IN_CH + 255) / 256;      // 4-channel chunks of a sample
    constexpr int OUT_CH = ROWS * COUT / 4, OUT_IT = (OUT_CH + 255) / 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    bf16_t* const img = reinterpret_cast<bf16_t*>(lds_raw);                   // [3 parts][PLANE]
    float* const oimg = reinterpret_cast<float*>(lds_raw);                    // the output image reuses the input images' LDS
    float* const red = reinterpret_cast<float*>(lds_raw + S::IMG_BYTES);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, half = lane >> 5;
    const int nb = wave % NB, kg = wave / NB;
    const int co = nb * 32 + m;

    auto ipos = [](int y, int x) { return ST == 2 ? (y * 2 + (x & 1)) * (G::W / 2) + (x >> 1) : y * G::W + x; };
    auto koff = [&](int ks) {
        const int tap = ks / CSI, cs = ks % CSI, ky = tap / KS, kx = tap % KS;
        return ipos(ky, kx) * PI + cs * 16;
    };

    int a_off[FRAGS];
#pragma unroll
    for (int f = 0; f < FRAGS; ++f) {
        const int r = min(f * 32 + m, ROWS - 1);          // rows past the map: a valid position, never stored
        a_off[f] = ipos((r / G::WO) * ST, (r % G::WO) * ST) * PI + half * 8;
    }

    float4 pin[IN_IT];
    auto prefetch_in = [&](int smp) __attribute__((always_inline)) {
        const float* base = in + (size_t)smp * (IN_POS * CIN);
#pragma unroll
        for (int i = 0; i < IN_IT; ++i) pin[i] = *reinterpret_cast<const float4*>(base + (size_t)min(tid + i * 256, IN_CH - 1) * 4);
    };
    int s = blockIdx.x;
    if (s >= ns) return;
    prefetch_in(s);
    __builtin_amdgcn_sched_barrier(0);                 // keep the sample's loads ahead of the weights'
    // requested after the first sample and in the order of use: the weights arrive while the sample is
    // split and written to LDS, and the first k-steps need not wait for the last weights
    bf16x8 bw[3][KPW];
#pragma unroll
    for (int i = 0; i < KPW; ++i)
#pragma unroll
        for (int p = 0; p < 3; ++p)
            bw[p][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(
                Wp + (size_t)p * WPLANE + ((size_t)(nb * KSTEPS + kg * KPW + i) * 64 + lane) * 8));
    const float bias_r = bias[co];

    for (; s < ns; s += gridDim.x) {
#pragma unroll
        for (int i = 0; i < IN_IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < IN_CH) {
                const int pos = ch / (CIN / 4), c4 = ch % (CIN / 4);
                uint2 hi, mid, lo;
                split3_pair(pin[i].x, pin[i].y, hi.x, mid.x, lo.x);
                split3_pair(pin[i].z, pin[i].w, hi.y, mid.y, lo.y);
                bf16_t* at = img + ipos(pos / G::W, pos % G::W) * PI + c4 * 4;
                *reinterpret_cast<uint2*>(at) = hi;
                *reinterpret_cast<uint2*>(at + PLANE) = mid;
                *reinterpret_cast<uint2*>(at + 2 * PLANE) = lo;
            }
        }
        __syncthreads();
        if (s + (int)gridDim.x < ns) prefetch_in(s + gridDim.x);

        f32x16 acc[FRAGS];
#pragma unroll
        for (int f = 0; f < FRAGS; ++f)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[f][q] = 0.f;
        // the fragments of step i + 1 are read while those of i are multiplied
        u32x4 a_cur[3][FRAGS], a_nxt[3][FRAGS];
        const int k0 = koff(kg * KPW);
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int f = 0; f < FRAGS; ++f) a_cur[p][f] = *reinterpret_cast<const u32x4*>(img + p * PLANE + a_off[f] + k0);
#pragma unroll
        for (int i = 0; i < KPW; ++i) {
            if (i + 1 < KPW) {
                const int kn = koff(kg * KPW + i + 1);
#pragma unroll
                for (int p = 0; p < 3; ++p)
#pragma unroll
                    for (int f = 0; f < FRAGS; ++f) a_nxt[p][f] = *reinterpret_cast<const u32x4*>(img + p * PLANE + a_off[f] + kn);
            }
            __builtin_amdgcn_sched_barrier(0);
            // smallest products first; consecutive MFMAs write different accumulators
            auto mul = [&](int pa, int pw) __attribute__((always_inline)) {
#pragma unroll
                for (int f = 0; f < FRAGS; ++f)
                    acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_cur[pa][f]), bw[pw][i], acc[f], 0, 0, 0);
            };
            mul(2, 0); mul(0, 2); mul(1, 1); mul(1, 0); mul(0, 1); mul(0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int f = 0; f < FRAGS; ++f) a_cur[p][f] = a_nxt[p][f];
        }
        if (kg > 0) {
#pragma unroll
            for (int f = 0; f < FRAGS; ++f)
#pragma unroll
                for (int q = 0; q < 16; ++q) red[((((kg - 1) * NB + nb) * FRAGS + f) * 16 + q) * 64 + lane] = acc[f][q];
        }
        __syncthreads();                               // the input images have been read by every wave
        if (kg == 0) {
#pragma unroll
            for (int g = 1; g < KW; ++g)
#pragma unroll
                for (int f = 0; f < FRAGS; ++f)
#pragma unroll
                    for (int q = 0; q < 16; ++q) acc[f][q] += red[((((g - 1) * NB + nb) * FRAGS + f) * 16 + q) * 64 + lane];
#pragma unroll
            for (int f = 0; f < FRAGS; ++f)
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int r = f * 32 + Mma<32>::row(q, lane);
                    if (r < ROWS) oimg[r * PO + co] = fmaxf(acc[f][q] + bias_r, 0.f);
                }
        }
        __syncthreads();                               // the output image is complete
        float* dst = out + (size_t)s * (ROWS * COUT);
#pragma unroll
        for (int i = 0; i < OUT_IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < OUT_CH) {
                const int pos = ch / (COUT / 4), c4 = ch % (COUT / 4);
                *reinterpret_cast<float4*>(dst + (size_t)ch * 4) = *reinterpret_cast<const float4*>(oimg + pos * PO + c4 * 4);
            }
        }
        __syncthreads();                               // the output image has been read: the next input may overwrite it
    }
}

template <class G>
inline hipError_t launch_conv_fwd_exact(hipStream_t s, const float* in, const bf16_t* Wp, const float* bias, float* out, int ns) {
    if (ns <= 0) return hipErrorInvalidValue;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        // more LDS than a kernel gets by default
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_fwd_exact_kernel<G>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, ConvFwdExactShape<G>::LDS_BYTES);
        if (e != hipSuccess) { cus = 0; return e; }
    }
    launch_k_lds((conv_fwd_exact_kernel<G>), dim3(std::min(ns, cus)), dim3(256), ConvFwdExactShape<G>::LDS_BYTES, s, in, Wp, bias, out, ns);
    return hipGetLastError();
}

}  // namespace paac
