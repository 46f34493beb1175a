// Forward pass of the convolutions of the fp32 path, one sample per workgroup from LDS, on the bf16
// matrix cores with exact operands.
//
// An fp32 number is the sum of three bf16 numbers (its 24 significand bits cut 8 + 8 + 8 by
// truncation); the product of two bf16 numbers is exact in fp32.  a*w = sum over the nine part
// products; the six of order >= 2^-16 are accumulated (the three left out are of relative size
// 2^-24 and below, the rounding level of an fp32 product), each one MFMA of four times the depth and
// twice the rate of the fp32 instruction.  The weights arrive already split, in the order in which
// the lanes read their B fragments (WeightSplits); the activations are split once, when a sample is
// written into LDS as three images.
//
// Layout and wave roles are those of the bf16 kernel (conv_fwd_direct_kernel): position-major images
// with the channels contiguous, de-interleaved by the parity of x for the stride-2 layer, pitch an odd
// multiple of 16 bytes; waves = (32-wide block of output channels) x (share of the k-steps), weights
// in registers, k-shares added through LDS, bias + ReLU results leave through an fp32 LDS image as
// contiguous 16-byte stores.
//
// Two kernels: conv_fwd_exact_kernel runs one layer (2 or 3) over any number of samples, a workgroup
// keeping its weights for all its samples; trunk_fwd_exact_kernel runs all convolutions of one sample
// in one workgroup (the first layer as in conv1_exact_kernel), for batches of at most one sample per
// compute unit: a layer's output is split into the next layer's LDS images directly, and is written to
// global memory only for the backward pass.
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

// Shape constants and the phases of one layer (2 or 3) for the 256 threads of a workgroup.
template <class G> struct ExactConv {
    static_assert((G::ST == 1 || G::ST == 2) && G::CIN % 16 == 0 && G::COUT % 32 == 0 && G::COUT <= 64, "layer shape");
    static_assert(G::ST == 1 || G::W % 2 == 0, "x parity planes");
    static constexpr int CIN = G::CIN, COUT = G::COUT, KS = G::KS, ST = G::ST;
    static constexpr int PI = CIN + 8, PO = COUT + 8;         // position pitches: bf16 input images, fp32 output image
    static constexpr int NB = COUT / 32, KW = 4 / NB, QW = 16 / KW;
    static constexpr int CSI = CIN / 16, KSTEPS = KS * KS * CSI, KPW = KSTEPS / KW;
    static_assert(KSTEPS % KW == 0, "equal k-shares");
    static constexpr int ROWS = G::HO * G::WO, FRAGS = (ROWS + 31) / 32;
    static constexpr int IN_POS = G::H * G::W, PLANE = IN_POS * PI;
    static constexpr int WPLANE = NB * 32 * G::KK;            // elements of one part of the weights
    static constexpr int IN_BYTES = 3 * PLANE * 2, OUT_BYTES = ROWS * PO * 4;
    static constexpr int IMG_BYTES = IN_BYTES > OUT_BYTES ? IN_BYTES : OUT_BYTES;
    static constexpr int RED_FLOATS = (KW - 1) * NB * FRAGS * 16 * 64;
    static constexpr int IN_CH = IN_POS * CIN / 4, IN_IT = (IN_CH + 255) / 256;       // 4-channel chunks of a sample
    static constexpr int OUT_CH = ROWS * COUT / 4, OUT_IT = (OUT_CH + 255) / 256;
    static_assert(IN_BYTES % 16 == 0 && OUT_BYTES % 16 == 0 && (PLANE * 2) % 16 == 0, "16-byte aligned images");

    // LDS position of input (y, x)
    static __device__ __forceinline__ constexpr int ipos(int y, int x) {
        return ST == 2 ? (y * 2 + (x & 1)) * (G::W / 2) + (x >> 1) : y * G::W + x;
    }
    // offset of k-step ks = (ky, kx, channel group) relative to a row's base
    static __device__ __forceinline__ constexpr int koff(int ks) {
        const int tap = ks / CSI, cs = ks % CSI, ky = tap / KS, kx = tap % KS;
        return ipos(ky, kx) * PI + cs * 16;
    }

    // this wave's share of the three weight parts, requested in the order of use
    static __device__ __forceinline__ void load_weights(const bf16_t* __restrict__ Wp, int nb, int kg, int lane, bf16x8 (&bw)[3][KPW]) {
#pragma unroll
        for (int i = 0; i < KPW; ++i)
#pragma unroll
            for (int p = 0; p < 3; ++p)
                bw[p][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(
                    Wp + (size_t)p * WPLANE + ((size_t)(nb * KSTEPS + kg * KPW + i) * 64 + lane) * 8));
    }

    // the three parts of k-step i of this wave's share
    static __device__ __forceinline__ void load_weights_step(const bf16_t* __restrict__ Wp, int nb, int kg, int lane, int i, bf16x8 (&bw)[3][KPW]) {
#pragma unroll
        for (int p = 0; p < 3; ++p)
            bw[p][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(
                Wp + (size_t)p * WPLANE + ((size_t)(nb * KSTEPS + kg * KPW + i) * 64 + lane) * 8));
    }

    static __device__ __forceinline__ void row_offsets(int lane, int (&a_off)[FRAGS]) {
        const int m = lane & 31, half = lane >> 5;
#pragma unroll
        for (int f = 0; f < FRAGS; ++f) {
            const int r = min(f * 32 + m, ROWS - 1);          // rows past the map: a valid position, never stored
            a_off[f] = ipos((r / G::WO) * ST, (r % G::WO) * ST) * PI + half * 8;
        }
    }

    // chunk ch (four channels of one position) of a sample -> its place in the three images
    static __device__ __forceinline__ void split_store(float4 v, int ch, bf16_t* img) {
        const int pos = ch / (CIN / 4), c4 = ch % (CIN / 4);
        uint2 hi, mid, lo;
        split3_pair(v.x, v.y, hi.x, mid.x, lo.x);
        split3_pair(v.z, v.w, hi.y, mid.y, lo.y);
        bf16_t* at = img + ipos(pos / G::W, pos % G::W) * PI + c4 * 4;
        *reinterpret_cast<uint2*>(at) = hi;
        *reinterpret_cast<uint2*>(at + PLANE) = mid;
        *reinterpret_cast<uint2*>(at + 2 * PLANE) = lo;
    }

    // acc += this wave's k-steps of (images) x (weights); the fragments of step i + 1 are read while
    // those of i are multiplied
    // `between(i)` runs after the MFMAs of step i have been issued (requests for later phases go there:
    // the matrix pipe is busy for hundreds of cycles, the memory instructions issue in its shadow).
    struct Nothing { __device__ __forceinline__ void operator()(int) const {} };
    template <class F = Nothing>
    static __device__ __forceinline__ void mfma(const bf16_t* img, const int (&a_off)[FRAGS], int kg, const bf16x8 (&bw)[3][KPW],
                                                f32x16 (&acc)[FRAGS], F&& between = F()) {
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
            between(i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int f = 0; f < FRAGS; ++f) a_cur[p][f] = a_nxt[p][f];
        }
    }

    // The k-shares of a column block are added and finished (bias + ReLU into the fp32 output image,
    // which may reuse the input images' LDS) by all of the block's waves, each taking QW of the 16
    // accumulator registers of every fragment; sums run in the fixed order own share, then the others
    // by wave.  Two barriers: the input images have been read by every wave / the output image is complete.
    static __device__ __forceinline__ void finish(const f32x16 (&acc)[FRAGS], float* red, float* oimg, int nb, int kg, int lane, float bias_r) {
        auto slot = [&](int dst, int src, int f, int qq) {
            return ((((dst * (KW - 1) + (src < dst ? src : src - 1)) * NB + nb) * FRAGS + f) * QW + qq) * 64 + lane;
        };
        // kg is wave-uniform but not a constant: one copy of the code per value keeps every accumulator
        // index a constant (a register array indexed at run time turns into long select chains)
        auto per_kg = [&](auto&& fn) __attribute__((always_inline)) {
            if (kg == 0) fn(std::integral_constant<int, 0>());
            if constexpr (KW > 1) { if (kg == 1) fn(std::integral_constant<int, 1>()); }
            if constexpr (KW > 2) {
                if (kg == 2) fn(std::integral_constant<int, 2>());
                if (kg == 3) fn(std::integral_constant<int, 3>());
            }
        };
        per_kg([&](auto KG) __attribute__((always_inline)) {
            constexpr int k = decltype(KG)::value;
#pragma unroll
            for (int g = 0; g < KW; ++g)
                if (g != k) {
#pragma unroll
                    for (int f = 0; f < FRAGS; ++f)
#pragma unroll
                        for (int qq = 0; qq < QW; ++qq) red[slot(g, k, f, qq)] = acc[f][g * QW + qq];
                }
        });
        __syncthreads();
        const int co = nb * 32 + (lane & 31);
        per_kg([&](auto KG) __attribute__((always_inline)) {
            constexpr int k = decltype(KG)::value;
#pragma unroll
            for (int f = 0; f < FRAGS; ++f)
#pragma unroll
                for (int qq = 0; qq < QW; ++qq) {
                    float v = acc[f][k * QW + qq];
#pragma unroll
                    for (int g = 0; g < KW; ++g)
                        if (g != k) v += red[slot(k, g, f, qq)];
                    const int r = f * 32 + Mma<32>::row(k * QW + qq, lane);
                    if (r < ROWS) oimg[r * PO + co] = fmaxf(v + bias_r, 0.f);
                }
        });
        __syncthreads();
    }
};

// ---------------------------------------------------------------------------------------------
// One layer, any number of samples.
template <class G>
__global__ __launch_bounds__(256, 1) void conv_fwd_exact_kernel(const float* __restrict__ in, const bf16_t* __restrict__ Wp,
                                                                const float* __restrict__ bias, float* __restrict__ out, int ns) {
    typedef ExactConv<G> S;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    bf16_t* const img = reinterpret_cast<bf16_t*>(lds_raw);                   // [3 parts][PLANE]
    float* const oimg = reinterpret_cast<float*>(lds_raw);                    // the output image reuses the input images' LDS
    float* const red = reinterpret_cast<float*>(lds_raw + S::IMG_BYTES);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nb = wave % S::NB, kg = wave / S::NB;

    int a_off[S::FRAGS];
    S::row_offsets(lane, a_off);

    float4 pin[S::IN_IT];
    auto prefetch_in = [&](int smp) __attribute__((always_inline)) {
        const float* base = in + (size_t)smp * (S::IN_POS * S::CIN);
#pragma unroll
        for (int i = 0; i < S::IN_IT; ++i) pin[i] = *reinterpret_cast<const float4*>(base + (size_t)min(tid + i * 256, S::IN_CH - 1) * 4);
    };
    int s = blockIdx.x;
    if (s >= ns) return;
    prefetch_in(s);
    __builtin_amdgcn_sched_barrier(0);                 // keep the sample's loads ahead of the weights'
    // the weights arrive while the sample is split and written to LDS
    bf16x8 bw[3][S::KPW];
    S::load_weights(Wp, nb, kg, lane, bw);
    const float bias_r = bias[nb * 32 + (lane & 31)];

    for (; s < ns; s += gridDim.x) {
        // (threads past the last chunk repeat it: a load that is used under a condition only would be
        // moved behind the weights' loads, and the split would wait for those as well)
#pragma unroll
        for (int i = 0; i < S::IN_IT; ++i) S::split_store(pin[i], min(tid + i * 256, S::IN_CH - 1), img);
        __syncthreads();
        if (s + (int)gridDim.x < ns) prefetch_in(s + gridDim.x);

        f32x16 acc[S::FRAGS];
#pragma unroll
        for (int f = 0; f < S::FRAGS; ++f)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[f][q] = 0.f;
        S::mfma(img, a_off, kg, bw, acc);
        S::finish(acc, red, oimg, nb, kg, lane, bias_r);
        float* dst = out + (size_t)s * (S::ROWS * S::COUT);
#pragma unroll
        for (int i = 0; i < S::OUT_IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < S::OUT_CH) {
                const int pos = ch / (S::COUT / 4), c4 = ch % (S::COUT / 4);
                *reinterpret_cast<float4*>(dst + (size_t)ch * 4) = *reinterpret_cast<const float4*>(oimg + pos * S::PO + c4 * 4);
            }
        }
        __syncthreads();                               // the output image has been read: the next input may overwrite it
    }
}

inline int device_cus() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    }
    return cus;
}

template <class G>
inline hipError_t launch_conv_fwd_exact(hipStream_t s, const float* in, const bf16_t* Wp, const float* bias, float* out, int ns) {
    if (ns <= 0) return hipErrorInvalidValue;
    constexpr int LDS = ExactConv<G>::IMG_BYTES + ExactConv<G>::RED_FLOATS * 4;
    static_assert(LDS <= 160 * 1024, "fits the LDS of a compute unit");
    static bool ready = false;
    if (!ready) {                       // more LDS than a kernel gets by default
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_fwd_exact_kernel<G>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        ready = true;
    }
    launch_k_lds((conv_fwd_exact_kernel<G>), dim3(std::min(ns, device_cus())), dim3(256), LDS, s, in, Wp, bias, out, ns);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// All convolutions of one sample in one workgroup.  G3 = NoLayer: two layers.
struct NoLayer {};
template <class G1, class G2, class G3> struct TrunkShape {
    static constexpr bool L3 = !std::is_same<G3, NoLayer>::value;
    typedef ExactConv<G2> S2;
    typedef ExactConv<std::conditional_t<L3, G3, G2>> S3;
    static constexpr int IMG1 = G1::CIN * G1::H * G1::W * 2;                  // the byte image as bf16
    // region A: layer 2's input images; later its output image, behind it layer 3's input images,
    // later layer 3's output image.  Region B: the first layer's image; later the k-share sums.
    static constexpr int OFF3 = S2::OUT_BYTES;
    static constexpr int A_NEED3 = OFF3 + (L3 ? S3::IN_BYTES : 0);
    static constexpr int A_BYTES = S2::IN_BYTES > A_NEED3 ? S2::IN_BYTES : A_NEED3;
    static constexpr int RED = (S2::RED_FLOATS > (L3 ? S3::RED_FLOATS : 0) ? S2::RED_FLOATS : S3::RED_FLOATS) * 4;
    static constexpr int B_BYTES = IMG1 > RED ? IMG1 : RED;
    static constexpr int LDS = A_BYTES + B_BYTES;
    static_assert(OFF3 % 16 == 0 && A_BYTES % 16 == 0 && IMG1 % 16 == 0, "16-byte aligned regions");
    static_assert(LDS <= 160 * 1024, "fits the LDS of a compute unit");
    static_assert(G1::HO == G2::H && G1::WO == G2::W && G1::COUT == G2::CIN && G2::CIN <= 32, "layer 1 feeds layer 2");
};

template <class G1, class G2, class G3>
__global__ __launch_bounds__(256, 1) void trunk_fwd_exact_kernel(const uint8_t* __restrict__ x, const bf16_t* __restrict__ W1p,
                                                                 const float* __restrict__ b1, float* __restrict__ out1,
                                                                 const bf16_t* __restrict__ W2p, const float* __restrict__ b2, float* __restrict__ out2,
                                                                 const bf16_t* __restrict__ W3p, const float* __restrict__ b3, float* __restrict__ out3,
                                                                 int ns, float scale) {
    typedef TrunkShape<G1, G2, G3> T;
    typedef typename T::S2 S2;
    typedef typename T::S3 S3;
    static_assert(G1::CIN == 4 && G1::H == 84 && G1::W == 84 && G1::KS == 8 && G1::ST == 4 && G1::COUT <= 32, "first layer");
    constexpr int PLANE1 = G1::H * G1::W, SAMPLE = 4 * PLANE1;
    constexpr int CHUNKS = SAMPLE / 16, IT = (CHUNKS + 255) / 256;
    constexpr int ROWS1 = G1::HO * G1::WO, FRAGS1 = (ROWS1 + 31) / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    bf16_t* const img2 = reinterpret_cast<bf16_t*>(lds_raw);
    float* const oimg2 = reinterpret_cast<float*>(lds_raw);
    bf16_t* const img3 = reinterpret_cast<bf16_t*>(lds_raw + T::OFF3);
    float* const oimg3 = reinterpret_cast<float*>(lds_raw);
    bf16_t* const img1 = reinterpret_cast<bf16_t*>(lds_raw + T::A_BYTES);
    float* const red = reinterpret_cast<float*>(lds_raw + T::A_BYTES);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fidx = lane & 31, half = lane >> 5;
    const int s = blockIdx.x;
    if (s >= ns) return;

    // ---- requests: the biases (in hand long before a wait could fall behind a store), the sample,
    // then the first layer's weights
    const int nb2 = wave % S2::NB, kg2 = wave / S2::NB;
    const int nb3 = wave % S3::NB, kg3 = wave / S3::NB;
    const float bias1 = fidx < G1::COUT ? b1[fidx] : 0.f;
    const float bias2 = b2[nb2 * 32 + fidx];
    float bias3 = 0.f;
    if constexpr (T::L3) bias3 = b3[nb3 * 32 + fidx];
    uint4 pre[IT];
#pragma unroll
    for (int i = 0; i < IT; ++i) pre[i] = *reinterpret_cast<const uint4*>(x + (size_t)s * SAMPLE + (size_t)min(tid + i * 256, CHUNKS - 1) * 16);
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 w1[3][16];
#pragma unroll
    for (int kt = 0; kt < 16; ++kt)
#pragma unroll
        for (int p = 0; p < 3; ++p)
            w1[p][kt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(W1p + p * 8192 + (kt * 64 + lane) * 8));
    __builtin_amdgcn_sched_barrier(0);

    // ---- first layer: bytes -> bf16 in the same linear order
    // (threads past the last chunk repeat it: a load that is used under a condition only would be
    // moved behind the weights' loads, and the conversion would wait for those as well)
#pragma unroll
    for (int i = 0; i < IT; ++i) {
        uint4* dst = reinterpret_cast<uint4*>(img1 + min(tid + i * 256, CHUNKS - 1) * 16);
        dst[0] = u8x8_to_bf16(make_uint2(pre[i].x, pre[i].y));
        dst[1] = u8x8_to_bf16(make_uint2(pre[i].z, pre[i].w));
    }
    __syncthreads();
    // Fragments wave, wave + 4, .. of the 32-position fragments, all at once (k-steps outside, fragments
    // inside: four independent accumulators per weight fragment; a fragment index past the map repeats
    // the last position and is not stored).  The second layer's weights are requested on the way, a
    // k-step's worth after each k-step: in the shadow of the MFMAs, and before the stores of this
    // layer's epilogue, so that waiting for them never waits for a store.
    constexpr int FPW = (FRAGS1 + 3) / 4;
    const bf16_t* a0[FPW];
    f32x16 acc1[FPW];
#pragma unroll
    for (int j = 0; j < FPW; ++j) {
        const int r = min((wave + 4 * j) * 32 + fidx, ROWS1 - 1);
        a0[j] = img1 + ((r / G1::WO) * G1::ST + half) * G1::W + (r % G1::WO) * G1::ST;
#pragma unroll
        for (int q = 0; q < 16; ++q) acc1[j][q] = 0.f;
    }
    bf16x8 w2[3][S2::KPW];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 a[FPW];
#pragma unroll
            for (int j = 0; j < FPW; ++j) {
                const uint2* ap = reinterpret_cast<const uint2*>(a0[j] + c * PLANE1 + ks * 2 * G1::W);   // 8-byte aligned
                const uint2 lo = ap[0], hi = ap[1];
                a[j] = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
            }
#pragma unroll
            for (int p = 2; p >= 0; --p)
#pragma unroll
                for (int j = 0; j < FPW; ++j) acc1[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], w1[p][c * 4 + ks], acc1[j], 0, 0, 0);
            // the second layer's weights, a few per k-step, in the shadow of the MFMAs just issued
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = (c * 4 + ks) * S2::KPW / 16; i < (c * 4 + ks + 1) * S2::KPW / 16; ++i)
                S2::load_weights_step(W2p, nb2, kg2, lane, i, w2);
            __builtin_amdgcn_sched_barrier(0);
        }
    // bias + ReLU, split into layer 2's images.  Lanes m and m ^ 1 hold neighbouring channels of one
    // position: one word per pair and part.
#pragma unroll
    for (int j = 0; j < FPW; ++j) {
        const int f = wave + 4 * j;
        if (f < FRAGS1) {
#pragma unroll
            for (int q = 0; q < 16; q += 2) {
                const float v0 = fmaxf(acc1[j][q] * scale + bias1, 0.f), v1 = fmaxf(acc1[j][q + 1] * scale + bias1, 0.f);
                const int r0 = f * 32 + Mma<32>::row(q, lane), r1 = f * 32 + Mma<32>::row(q + 1, lane);
                const float p0 = lane_xor1(v0), p1 = lane_xor1(v1);
                const bool odd = fidx & 1;
                const int rr = odd ? r1 : r0;
                unsigned hi, mid, lo;
                split3_pair(odd ? p1 : v0, odd ? v1 : p0, hi, mid, lo);
                if (rr < ROWS1 && fidx < G1::COUT) {
                    bf16_t* at = img2 + S2::ipos(rr / G1::WO, rr % G1::WO) * S2::PI + (fidx & ~1);
                    *reinterpret_cast<unsigned*>(at) = hi;
                    *reinterpret_cast<unsigned*>(at + S2::PLANE) = mid;
                    *reinterpret_cast<unsigned*>(at + 2 * S2::PLANE) = lo;
                }
            }
        }
    }
    __syncthreads();                                   // layer 2's images are complete, the first image is free
    // The first layer's output goes to global memory (the backward pass reads it) from the images:
    // hi + mid + lo is the fp32 value again, and a thread stores four channels at once (stores of
    // single values straight from the accumulator layout are eight times as many instructions).
    {
        constexpr int O1_CH = ROWS1 * G1::COUT / 4;
        float* const o1 = out1 + (size_t)s * (ROWS1 * G1::COUT);
#pragma unroll
        for (int i = 0; i < (O1_CH + 255) / 256; ++i) {
            const int ch = tid + i * 256;
            if (ch < O1_CH) {
                const int pos = ch / (G1::COUT / 4), c4 = ch % (G1::COUT / 4);
                const bf16_t* at = img2 + S2::ipos(pos / G1::WO, pos % G1::WO) * S2::PI + c4 * 4;
                const uint2 h = *reinterpret_cast<const uint2*>(at), m = *reinterpret_cast<const uint2*>(at + S2::PLANE),
                            l = *reinterpret_cast<const uint2*>(at + 2 * S2::PLANE);
                auto lo16 = [](unsigned w) { return __uint_as_float(w << 16); };
                auto hi16 = [](unsigned w) { return __uint_as_float(w & 0xffff0000u); };
                float4 v;
                v.x = (lo16(h.x) + lo16(m.x)) + lo16(l.x); v.y = (hi16(h.x) + hi16(m.x)) + hi16(l.x);
                v.z = (lo16(h.y) + lo16(m.y)) + lo16(l.y); v.w = (hi16(h.y) + hi16(m.y)) + hi16(l.y);
                *reinterpret_cast<float4*>(o1 + (size_t)ch * 4) = v;
            }
        }
    }

    // ---- second layer
    int a_off2[S2::FRAGS];
    S2::row_offsets(lane, a_off2);
    f32x16 acc2[S2::FRAGS];
#pragma unroll
    for (int f = 0; f < S2::FRAGS; ++f)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc2[f][q] = 0.f;
    // the third layer's weights are requested k-step by k-step while the second layer multiplies
    // (its own weights' registers become free at the same rate)
    bf16x8 w3[3][S3::KPW];
    S2::mfma(img2, a_off2, kg2, w2, acc2, [&](int i) __attribute__((always_inline)) {
        if constexpr (T::L3) {
#pragma unroll
            for (int j = 0; j < S3::KPW; ++j)
                if (j * S2::KPW / S3::KPW == i) S3::load_weights_step(W3p, nb3, kg3, lane, j, w3);
        }
    });
    __builtin_amdgcn_sched_barrier(0);
    S2::finish(acc2, red, oimg2, nb2, kg2, lane, bias2);
    float* const o2 = out2 + (size_t)s * (S2::ROWS * S2::COUT);
#pragma unroll
    for (int i = 0; i < S2::OUT_IT; ++i) {
        const int ch = tid + i * 256;
        if (ch < S2::OUT_CH) {
            const int pos = ch / (S2::COUT / 4), c4 = ch % (S2::COUT / 4);
            const float4 v = *reinterpret_cast<const float4*>(oimg2 + pos * S2::PO + c4 * 4);
            *reinterpret_cast<float4*>(o2 + (size_t)ch * 4) = v;
            if constexpr (T::L3) S3::split_store(v, ch, img3);       // layer 2's output order is layer 3's input order
        }
    }
    if constexpr (T::L3) {
        static_assert(G2::HO == G3::H && G2::WO == G3::W && G2::COUT == G3::CIN && G3::ST == 1, "layer 2 feeds layer 3");
        __syncthreads();                               // layer 3's images are complete
        int a_off3[S3::FRAGS];
        S3::row_offsets(lane, a_off3);
        f32x16 acc3[S3::FRAGS];
#pragma unroll
        for (int f = 0; f < S3::FRAGS; ++f)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc3[f][q] = 0.f;
        S3::mfma(img3, a_off3, kg3, w3, acc3);
        S3::finish(acc3, red, oimg3, nb3, kg3, lane, bias3);
        float* const o3 = out3 + (size_t)s * (S3::ROWS * S3::COUT);
#pragma unroll
        for (int i = 0; i < S3::OUT_IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < S3::OUT_CH) {
                const int pos = ch / (S3::COUT / 4), c4 = ch % (S3::COUT / 4);
                *reinterpret_cast<float4*>(o3 + (size_t)ch * 4) = *reinterpret_cast<const float4*>(oimg3 + pos * S3::PO + c4 * 4);
            }
        }
    }
}

// ns <= compute units (one workgroup per sample, no loop over samples)
template <class G1, class G2, class G3>
inline hipError_t launch_trunk_fwd_exact(hipStream_t s, const uint8_t* x, const bf16_t* W1p, const float* b1, float* out1,
                                         const bf16_t* W2p, const float* b2, float* out2,
                                         const bf16_t* W3p, const float* b3, float* out3, int ns) {
    if (ns <= 0 || ns > device_cus()) return hipErrorInvalidValue;
    constexpr int LDS = TrunkShape<G1, G2, G3>::LDS;
    static bool ready = false;
    if (!ready) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(trunk_fwd_exact_kernel<G1, G2, G3>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        ready = true;
    }
    launch_k_lds((trunk_fwd_exact_kernel<G1, G2, G3>), dim3(ns), dim3(256), LDS, s, x, W1p, b1, out1, W2p, b2, out2, W3p, b3, out3, ns,
                 1.0f / 255.0f);
    return hipGetLastError();
}

}  // namespace paac
