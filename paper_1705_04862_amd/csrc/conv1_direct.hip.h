// First convolution (8x8, stride 4, uint8 NCHW input) with bf16 operands, straight from the image.
//
// The im2col view repeats every input byte in four output windows, and turning bytes into bf16 is
// the dominant cost of this layer in the generic GEMM kernel.  Here a workgroup takes NS consecutive
// samples at a time: their NS x 4 x 84 x 84 bytes are one contiguous block of global memory,
// loaded with 16-byte loads, converted ONCE and kept in LDS as bf16 in the same (c, y, x) order.
// The MFMA A fragment of an output position (oy, ox) and k-group (c, ky) is then the 16 bytes at
//   img[c][4*oy + ky][4*ox .. 4*ox + 7],
// i.e. one base address per fragment plus compile-time offsets; the weights (COUT x 256) stay in
// registers for the lifetime of the workgroup (read from a copy in fragment order).  An image row is 84 elements = 42 words: the rows of
// consecutive output rows continue each other's bank sequence, no padding is needed.
// NS = 1 (56 KB of LDS) lets two workgroups share a compute unit, so that one converts and waits
// while the other multiplies; its 400 output rows are 12.5 fragments of 32 (the last is half empty).
#pragma once
#include "gemm_bf16.hip.h"

namespace paac {

template <class G, int NS>
__global__ __launch_bounds__(256, 2) void conv1_direct_kernel(const uint8_t* __restrict__ x, const bf16_t* __restrict__ Wt,
                                                           const float* __restrict__ bias, bf16_t* __restrict__ out, int ns,
                                                           float scale) {
    static_assert(G::CIN == 4 && G::H == 84 && G::W == 84 && G::KS == 8 && G::ST == 4 && G::COUT <= 32, "first layer");
    constexpr int SAMPLE = G::CIN * G::H * G::W;            // 28224 bytes, a multiple of 16
    constexpr int CHUNKS = NS * SAMPLE / 16, IT = (CHUNKS + 255) / 256;
    constexpr int ROWS = G::HO * G::WO;                     // 400 output positions per sample
    constexpr int FRAGS = (NS * ROWS + 31) / 32;
    static_assert(SAMPLE % 16 == 0, "whole 16-byte chunks");
    __shared__ __attribute__((aligned(16))) bf16_t img[NS * SAMPLE];
    constexpr int LDS_O = G::COUT + 8, CPR = G::COUT / 8;     // staging row pitch (bf16), 16-byte chunks per output row
    __shared__ __attribute__((aligned(16))) bf16_t stage[4 * 32 * LDS_O];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fidx = lane & 31, kg = lane >> 5;
    const int pairs = (ns + NS - 1) / NS;                   // groups of NS samples
    const long total_bytes = (long)ns * SAMPLE;

    // weights of output channel fidx: sixteen k-steps of 16, this lane's eight k of each; the copy is laid
    // out [k/8][32 channels][8] (channels past COUT zero), so a wave reads one contiguous KB per k-step
    bf16x8 breg[16];
#pragma unroll
    for (int kt = 0; kt < 16; ++kt) breg[kt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Wt + (kt * 64 + lane) * 8));
    const float bias_r = fidx < G::COUT ? bias[fidx] : 0.f;

    uint4 pre[IT];
    auto prefetch = [&](int p) __attribute__((always_inline)) {
        const long base = (long)p * (NS * SAMPLE);
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            const int ch = tid + i * 256;
            const long off = base + (long)ch * 16;
            const bool ok = ch < CHUNKS && off < total_bytes;           // sample sizes are multiples of 16
            pre[i] = *reinterpret_cast<const uint4*>(x + (ok ? off : 0));
            if (!ok) pre[i] = zero_u4();
        }
    };
    int p = blockIdx.x;
    if (p >= pairs) return;
    prefetch(p);
    for (; p < pairs; p += gridDim.x) {
        // bytes -> bf16, same linear order
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            const int ch = tid + i * 256;
            if (ch < CHUNKS) {
                uint4* dst = reinterpret_cast<uint4*>(img + ch * 16);
                dst[0] = u8x8_to_bf16(make_uint2(pre[i].x, pre[i].y));
                dst[1] = u8x8_to_bf16(make_uint2(pre[i].z, pre[i].w));
            }
        }
        __syncthreads();
        if (p + (int)gridDim.x < pairs) prefetch(p + gridDim.x);       // in flight during the MFMA phase
        const int row0 = p * (NS * ROWS), M = ns * ROWS;
        for (int f = wave; f < FRAGS; f += 4) {
            const int row = min(f * 32 + fidx, NS * ROWS - 1);        // rows past the group: a valid address, never stored
            const int s = row / ROWS, r = row % ROWS, oy = r / G::WO, ox = r % G::WO;
            const bf16_t* a0 = img + s * SAMPLE + (oy * G::ST + kg) * G::W + ox * G::ST;
            f32x16 acc;
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[q] = 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const uint2* ap = reinterpret_cast<const uint2*>(a0 + c * (G::H * G::W) + ks * 2 * G::W);   // 8-byte aligned
                    const uint2 lo = ap[0], hi = ap[1];
                    const bf16x8 a = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, breg[c * 4 + ks], acc, 0, 0, 0);
                }
            // the fragment's 32 rows are one contiguous piece of the output: through a wave-private LDS
            // staging area it leaves as 16-byte stores instead of sixteen 2-byte stores per lane
            bf16_t* st = stage + wave * (32 * LDS_O);
            if (fidx < G::COUT) {
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    st[Mma<32>::row(q, lane) * LDS_O + fidx] = f2bf(fmaxf(acc[q] * scale + bias_r, 0.f));
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int c = 0; c < (32 * CPR + 63) / 64; ++c) {
                const int ch = lane + c * 64, lrow = ch / CPR, c8 = ch % CPR;
                const int lr = f * 32 + lrow, orow = row0 + lr;
                if (ch < 32 * CPR && lr < NS * ROWS && orow < M)
                    *reinterpret_cast<uint4*>(out + (size_t)orow * G::COUT + c8 * 8) = *reinterpret_cast<const uint4*>(st + lrow * LDS_O + c8 * 8);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();                                              // the image is rewritten next
    }
}

// The same layer for batches of at most one sample per compute unit: a workgroup takes one band of
// HO / PARTS output rows of one sample (its 4 x (4 BR + 4) image rows are four contiguous pieces of
// global memory), so that a compute unit holds two workgroups again and one loads and converts while the
// other multiplies.  Same order of MFMAs per output element as conv1_direct_kernel: the same bits.
template <class G, int PARTS>
__global__ __launch_bounds__(256, 2) void conv1_direct_band_kernel(const uint8_t* __restrict__ x, const bf16_t* __restrict__ Wt,
                                                                const float* __restrict__ bias, bf16_t* __restrict__ out, int ns,
                                                                float scale) {
    static_assert(G::CIN == 4 && G::H == 84 && G::W == 84 && G::KS == 8 && G::ST == 4 && G::COUT <= 32, "first layer");
    static_assert(G::HO % PARTS == 0, "bands of whole output rows");
    constexpr int SAMPLE = G::CIN * G::H * G::W, PLANE = G::H * G::W;
    constexpr int BR = G::HO / PARTS, IR = 4 * BR + 4;            // output rows per band, image rows it reads
    constexpr int CPC = IR * G::W / 16, CHUNKS = 4 * CPC, IT = (CHUNKS + 255) / 256;   // 16-byte chunks per channel piece
    constexpr int ROWS = BR * G::WO, FRAGS = (ROWS + 31) / 32;
    static_assert((IR * G::W) % 16 == 0 && (G::ST * G::W * BR) % 16 == 0 && PLANE % 16 == 0, "whole 16-byte chunks");
    __shared__ __attribute__((aligned(16))) bf16_t img[4 * IR * G::W];
    constexpr int LDS_O = G::COUT + 8, CPR = G::COUT / 8;     // staging row pitch (bf16), 16-byte chunks per output row
    __shared__ __attribute__((aligned(16))) bf16_t stage[4 * 32 * LDS_O];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fidx = lane & 31, kg = lane >> 5;
    const int items = ns * PARTS;

    uint4 pre[IT];
    auto prefetch = [&](int p) __attribute__((always_inline)) {
        const size_t base = (size_t)(p / PARTS) * SAMPLE + (size_t)(p % PARTS) * (BR * G::ST * G::W);
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            const int ch = tid + i * 256;
            const int cc = ch < CHUNKS ? ch : 0;
            pre[i] = *reinterpret_cast<const uint4*>(x + base + (size_t)(cc / CPC) * PLANE + (size_t)(cc % CPC) * 16);
        }
    };
    int p = blockIdx.x;
    if (p >= items) return;
    prefetch(p);
    bf16x8 breg[16];
#pragma unroll
    for (int kt = 0; kt < 16; ++kt) breg[kt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Wt + (kt * 64 + lane) * 8));
    const float bias_r = fidx < G::COUT ? bias[fidx] : 0.f;

    for (; p < items; p += gridDim.x) {
#pragma unroll
        for (int i = 0; i < IT; ++i) {                                // bytes -> bf16, same linear order
            const int ch = tid + i * 256;
            if (ch < CHUNKS) {
                uint4* dst = reinterpret_cast<uint4*>(img + ch * 16);
                dst[0] = u8x8_to_bf16(make_uint2(pre[i].x, pre[i].y));
                dst[1] = u8x8_to_bf16(make_uint2(pre[i].z, pre[i].w));
            }
        }
        __syncthreads();
        if (p + (int)gridDim.x < items) prefetch(p + gridDim.x);     // in flight during the MFMA phase
        const size_t orow0 = (size_t)(p / PARTS) * (G::HO * G::WO) + (size_t)(p % PARTS) * ROWS;
        for (int f = wave; f < FRAGS; f += 4) {
            const int r = min(f * 32 + fidx, ROWS - 1);               // rows past the band: a valid address, never stored
            const int oy = r / G::WO, ox = r % G::WO;
            const bf16_t* a0 = img + (oy * G::ST + kg) * G::W + ox * G::ST;
            f32x16 acc;
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[q] = 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const uint2* ap = reinterpret_cast<const uint2*>(a0 + c * (IR * G::W) + ks * 2 * G::W);   // 8-byte aligned
                    const uint2 lo = ap[0], hi = ap[1];
                    const bf16x8 a = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, breg[c * 4 + ks], acc, 0, 0, 0);
                }
            // the band's rows are one contiguous piece of the output: 16-byte stores through a wave-private staging area
            bf16_t* st = stage + wave * (32 * LDS_O);
            if (fidx < G::COUT) {
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    st[Mma<32>::row(q, lane) * LDS_O + fidx] = f2bf(fmaxf(acc[q] * scale + bias_r, 0.f));
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int c = 0; c < (32 * CPR + 63) / 64; ++c) {
                const int ch = lane + c * 64, lrow = ch / CPR, c8 = ch % CPR;
                const int lr = f * 32 + lrow;
                if (ch < 32 * CPR && lr < ROWS)
                    *reinterpret_cast<uint4*>(out + (orow0 + lr) * G::COUT + c8 * 8) = *reinterpret_cast<const uint4*>(st + lrow * LDS_O + c8 * 8);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();                                              // the image is rewritten next
    }
}

template <class G, int NS = 1>
inline hipError_t launch_conv1_direct(hipStream_t s, const uint8_t* x, const bf16_t* Wt, const float* bias, bf16_t* out, int ns) {
    if (ns <= 0) return hipErrorInvalidValue;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    }
    // up to half a sample per compute unit: four bands per sample, so that every compute unit still gets two
    // workgroups (select call at n_e = 32: 6.8 -> 4.7 us, n_e = 128: 7.6 -> 6.3 us; from 256 samples the step gains nothing)
    if (ns * 2 <= cus) {
        launch_k((conv1_direct_band_kernel<G, 4>), dim3(ns * 4), dim3(256), s, x, Wt, bias, out, ns, 1.0f / 255.0f);
        return hipGetLastError();
    }
    const int groups = (ns + NS - 1) / NS;
    launch_k((conv1_direct_kernel<G, NS>), dim3(std::min(groups, 2 * cus)), dim3(256), s, x, Wt, bias, out, ns, 1.0f / 255.0f);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// The same layer for the fp32 path, on the bf16 matrix cores without giving up fp32 accuracy.
// A byte (0..255) is exact in bf16, and an fp32 weight is exactly the sum of three bf16 numbers
// (its 24 significand bits cut into 8 + 8 + 8 by truncation: w = hi + mid + lo, every residual
// exact).  Every product byte x part is exact in fp32, so three bf16 MFMAs accumulate, in fp32,
// exactly the terms of the fp32 dot product; only the order of the fp32 additions differs from
// the fp32 MFMA path.  16 k per 32-cycle instruction x 3 parts against 2 k per 64-cycle fp32
// instruction: 5.3 times fewer matrix-core cycles, and no im2col gather.
// A workgroup takes one band of HO / PARTS output rows of one sample: its 4 x (4 BR + 4) image
// rows are four contiguous pieces of global memory.  The weights arrive as their three bf16 parts in
// fragment order (WeightSplits: the optimiser writes them with every update), 16 bytes per lane and k-step.
template <class G, int PARTS>
__global__ __launch_bounds__(256, 1) void conv1_exact_kernel(const uint8_t* __restrict__ x, const bf16_t* __restrict__ Wp,
                                                          const float* __restrict__ bias, float* __restrict__ out, int ns,
                                                          float scale) {
    static_assert(G::CIN == 4 && G::H == 84 && G::W == 84 && G::KS == 8 && G::ST == 4 && G::COUT <= 32, "first layer");
    static_assert(G::HO % PARTS == 0, "bands of whole output rows");
    constexpr int SAMPLE = G::CIN * G::H * G::W, PLANE = G::H * G::W;
    constexpr int BR = G::HO / PARTS, IR = 4 * BR + 4;            // output rows per band, image rows it reads
    constexpr int CPC = IR * G::W / 16, CHUNKS = 4 * CPC, IT = (CHUNKS + 255) / 256;   // 16-byte chunks per channel piece
    constexpr int ROWS = BR * G::WO, FRAGS = (ROWS + 31) / 32;
    static_assert((IR * G::W) % 16 == 0 && (G::ST * G::W * BR) % 16 == 0 && PLANE % 16 == 0, "whole 16-byte chunks");
    __shared__ __attribute__((aligned(16))) bf16_t img[4 * IR * G::W];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fidx = lane & 31, kg = lane >> 5;
    const int items = ns * PARTS;

    uint4 pre[IT];
    auto prefetch = [&](int p) __attribute__((always_inline)) {
        const size_t base = (size_t)(p / PARTS) * SAMPLE + (size_t)(p % PARTS) * (BR * G::ST * G::W);
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            const int ch = tid + i * 256;
            const bool ok = ch < CHUNKS;
            const int cc = ok ? ch : 0;
            pre[i] = *reinterpret_cast<const uint4*>(x + base + (size_t)(cc / CPC) * PLANE + (size_t)(cc % CPC) * 16);
        }
    };
    int p = blockIdx.x;
    if (p >= items) return;
    prefetch(p);

    // weights of output channel fidx, this lane's eight k of each of the sixteen k-steps, as three bf16 parts
    bf16x8 bh[16], bm[16], bl[16];
#pragma unroll
    for (int kt = 0; kt < 16; ++kt) {
        const bf16_t* w = Wp + (kt * 64 + lane) * 8;                // one contiguous KB per wave; channels COUT..31 are zero
        bh[kt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(w));
        bm[kt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(w + 8192));
        bl[kt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(w + 2 * 8192));
    }
    const float bias_r = fidx < G::COUT ? bias[fidx] : 0.f;

    for (; p < items; p += gridDim.x) {
#pragma unroll
        for (int i = 0; i < IT; ++i) {                                // bytes -> bf16, same linear order
            const int ch = tid + i * 256;
            if (ch < CHUNKS) {
                uint4* dst = reinterpret_cast<uint4*>(img + ch * 16);
                dst[0] = u8x8_to_bf16(make_uint2(pre[i].x, pre[i].y));
                dst[1] = u8x8_to_bf16(make_uint2(pre[i].z, pre[i].w));
            }
        }
        __syncthreads();
        if (p + (int)gridDim.x < items) prefetch(p + gridDim.x);     // in flight during the MFMA phase
        const size_t orow0 = (size_t)(p / PARTS) * (G::HO * G::WO) + (size_t)(p % PARTS) * ROWS;
        for (int f = wave; f < FRAGS; f += 4) {
            const int r = min(f * 32 + fidx, ROWS - 1);               // rows past the band: a valid address, never stored
            const int oy = r / G::WO, ox = r % G::WO;
            const bf16_t* a0 = img + (oy * G::ST + kg) * G::W + ox * G::ST;
            f32x16 acc;
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[q] = 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const uint2* ap = reinterpret_cast<const uint2*>(a0 + c * (IR * G::W) + ks * 2 * G::W);   // 8-byte aligned
                    const uint2 lo = ap[0], hi = ap[1];
                    const bf16x8 a = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bl[c * 4 + ks], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bm[c * 4 + ks], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bh[c * 4 + ks], acc, 0, 0, 0);
                }
            if (fidx < G::COUT) {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int lr = f * 32 + Mma<32>::row(q, lane);
                    if (lr < ROWS) out[(orow0 + lr) * G::COUT + fidx] = fmaxf(acc[q] * scale + bias_r, 0.f);
                }
            }
        }
        __syncthreads();                                              // the image is rewritten next
    }
}

// The same for small batches (a quarter or a tenth of a sample per workgroup, one item each): a wave that takes
// whole fragments needs all 48 KB of weight parts for 48 MFMAs, and loading them is what the kernel
// then waits for.  Here wave c takes input channel c (a quarter of the k-steps, 12 KB of weights) for
// all fragments of the band (four, or two with ten bands); the four partial sums of a fragment meet in LDS,
// every wave finishing a quarter of the band's accumulator registers (own share first, then the others by
// wave: a fixed order).
template <class G, int PARTS>
__global__ __launch_bounds__(256, 1) void conv1_exact_ksplit_kernel(const uint8_t* __restrict__ x, const bf16_t* __restrict__ Wp,
                                                                    const float* __restrict__ bias, float* __restrict__ out, int ns,
                                                                    float scale) {
    static_assert(G::CIN == 4 && G::H == 84 && G::W == 84 && G::KS == 8 && G::ST == 4 && G::COUT <= 32, "first layer");
    static_assert(G::HO % PARTS == 0, "bands of whole output rows");
    constexpr int SAMPLE = G::CIN * G::H * G::W, PLANE = G::H * G::W;
    constexpr int BR = G::HO / PARTS, IR = 4 * BR + 4;
    constexpr int CPC = IR * G::W / 16, CHUNKS = 4 * CPC, IT = (CHUNKS + 255) / 256;
    constexpr int ROWS = BR * G::WO, FRAGS = (ROWS + 31) / 32;
    // the band's FRAGS x 16 accumulator registers are finished in four units, one per wave: unit u is
    // fragment u % FRAGS, registers (u / FRAGS) RPU .. + RPU (a whole fragment with four fragments, half of one with two)
    static_assert(FRAGS == 4 || FRAGS == 2, "four finishing units of whole or half fragments");
    constexpr int RPU = 16 * FRAGS / 4;
    static_assert((IR * G::W) % 16 == 0 && (G::ST * G::W * BR) % 16 == 0 && PLANE % 16 == 0, "whole 16-byte chunks");
    __shared__ __attribute__((aligned(16))) bf16_t img[4 * IR * G::W];
    __shared__ float red[4 * 3 * RPU * 64];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fidx = lane & 31, kg = lane >> 5;
    const int p = blockIdx.x;
    if (p >= ns * PARTS) return;
    const float bias_r = fidx < G::COUT ? bias[fidx] : 0.f;

    // the band's image (threads past the last chunk repeat it: no load is used under a condition only)
    const size_t base = (size_t)(p / PARTS) * SAMPLE + (size_t)(p % PARTS) * (BR * G::ST * G::W);
    uint4 pre[IT];
#pragma unroll
    for (int i = 0; i < IT; ++i) {
        const int cc = min(tid + i * 256, CHUNKS - 1);
        pre[i] = *reinterpret_cast<const uint4*>(x + base + (size_t)(cc / CPC) * PLANE + (size_t)(cc % CPC) * 16);
    }
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 w[3][4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int q = 0; q < 3; ++q)
            w[q][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Wp + q * 8192 + ((wave * 4 + ks) * 64 + lane) * 8));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < IT; ++i) {
        uint4* dst = reinterpret_cast<uint4*>(img + min(tid + i * 256, CHUNKS - 1) * 16);
        dst[0] = u8x8_to_bf16(make_uint2(pre[i].x, pre[i].y));
        dst[1] = u8x8_to_bf16(make_uint2(pre[i].z, pre[i].w));
    }
    __syncthreads();

    const bf16_t* a0[FRAGS];
    f32x16 acc[FRAGS];
#pragma unroll
    for (int f = 0; f < FRAGS; ++f) {
        const int r = min(f * 32 + fidx, ROWS - 1);               // rows past the band: a valid address, never stored
        a0[f] = img + wave * (IR * G::W) + ((r / G::WO) * G::ST + kg) * G::W + (r % G::WO) * G::ST;
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[f][q] = 0.f;
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        bf16x8 a[FRAGS];
#pragma unroll
        for (int f = 0; f < FRAGS; ++f) {
            const uint2* ap = reinterpret_cast<const uint2*>(a0[f] + ks * 2 * G::W);   // 8-byte aligned
            const uint2 lo = ap[0], hi = ap[1];
            a[f] = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
        }
#pragma unroll
        for (int q = 2; q >= 0; --q)
#pragma unroll
            for (int f = 0; f < FRAGS; ++f) acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], w[q][ks], acc[f], 0, 0, 0);
    }
    // one copy of the exchange per wave keeps every accumulator index a constant
    auto per_wave = [&](auto&& fn) __attribute__((always_inline)) {
        if (wave == 0) fn(std::integral_constant<int, 0>());
        if (wave == 1) fn(std::integral_constant<int, 1>());
        if (wave == 2) fn(std::integral_constant<int, 2>());
        if (wave == 3) fn(std::integral_constant<int, 3>());
    };
    auto slot = [&](int dst, int src, int q) { return ((dst * 3 + (src < dst ? src : src - 1)) * RPU + q) * 64 + lane; };
    per_wave([&](auto WV) __attribute__((always_inline)) {
        constexpr int wv = decltype(WV)::value;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (u != wv) {
#pragma unroll
                for (int q = 0; q < RPU; ++q) red[slot(u, wv, q)] = acc[u % FRAGS][(u / FRAGS) * RPU + q];
            }
    });
    __syncthreads();
    const size_t orow0 = (size_t)(p / PARTS) * (G::HO * G::WO) + (size_t)(p % PARTS) * ROWS;
    per_wave([&](auto WV) __attribute__((always_inline)) {
        constexpr int wv = decltype(WV)::value;
        constexpr int f = wv % FRAGS, q0 = (wv / FRAGS) * RPU;
#pragma unroll
        for (int q = 0; q < RPU; ++q) {
            float v = acc[f][q0 + q];
#pragma unroll
            for (int g = 0; g < 4; ++g)
                if (g != wv) v += red[slot(wv, g, q)];
            const int lr = f * 32 + Mma<32>::row(q0 + q, lane);
            if (fidx < G::COUT && lr < ROWS) out[(orow0 + lr) * G::COUT + fidx] = fmaxf(v * scale + bias_r, 0.f);
        }
    });
}

template <class G, int PARTS>
inline void launch_conv1_exact_p(hipStream_t s, int cus, const uint8_t* x, const bf16_t* Wk, const float* bias, float* out, int ns) {
    launch_k((conv1_exact_kernel<G, PARTS>), dim3(std::min(ns * PARTS, 2 * cus)), dim3(256), s, x, Wk, bias, out, ns, 1.0f / 255.0f);
}

template <class G>
inline hipError_t launch_conv1_exact(hipStream_t s, const uint8_t* x, const bf16_t* Wk, const float* bias, float* out, int ns) {
    if (ns <= 0) return hipErrorInvalidValue;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    }
    // one workgroup per compute unit (its registers allow no more): split samples into bands while
    // that still gives every workgroup a compute unit of its own
    const int parts = ns * 4 <= cus ? 4 : (ns * 2 <= cus ? 2 : 1);
    // up to a fifth of a sample per compute unit: ten bands of two output rows (two fragments, each finished in
    // halves), two workgroups per compute unit (n_e = 32: 5.85 -> 5.5 us per select call, n_e = 4: 5.0 -> 4.35 us)
    if (ns * 10 <= 2 * cus) launch_k((conv1_exact_ksplit_kernel<G, 10>), dim3(ns * 10), dim3(256), s, x, Wk, bias, out, ns, 1.0f / 255.0f);
    else if (parts == 4) launch_k((conv1_exact_ksplit_kernel<G, 4>), dim3(ns * 4), dim3(256), s, x, Wk, bias, out, ns, 1.0f / 255.0f);
    else if (parts == 2) launch_conv1_exact_p<G, 2>(s, cus, x, Wk, bias, out, ns);
    else launch_conv1_exact_p<G, 1>(s, cus, x, Wk, bias, out, ns);
    return hipGetLastError();
}

}  // namespace paac
