// Weight gradient of the first convolution (8x8, stride 4, uint8 NCHW input), straight from the image.
//
//   dW[k = (c, ky, kx)][co] = sum over (sample, oy, ox) of  x[c][4 oy + ky][4 ox + kx] * dY[oy][ox][co]
//
// As an MFMA the reduction index is the output position, so the A operand wants, for one (c, ky, kx),
// the pixels of eight consecutive ox: every fourth byte of an image row.  The image band of a work
// item is therefore kept in LDS de-interleaved by x mod 4 ("phase"): row (c, y, phase) holds
// x = phase, phase + 4, ...  and eight consecutive ox are sixteen contiguous bytes.  kx >= 4 starts one
// element later; a second copy of the band, shifted by one element, keeps those reads 16-byte aligned.
// dY is kept transposed, [co][position slot], so that the B operand (eight positions of one output
// channel) is contiguous as well; an output row takes 24 slots (20 positions + 4 zeros) = three
// groups of eight, a band of five output rows 15 groups + one zero group = eight 16-wide k-steps.
//
// A work item is one band of one sample; a workgroup walks over items with a stride of the grid and
// keeps its 256 x 32 accumulators (wave w: input channel w, two blocks of four ky) in registers
// until the end, when it writes one partial dW [256][COUT] and one partial db [COUT] (the bias
// gradient is the sum of dY over positions, accumulated from the values as they are loaded).
// The partials are summed by the gradient reduction in a fixed order.
//
// EXACT = true serves the fp32 path: bytes are exact in bf16 and dY (fp32) is cut into three bf16
// parts whose sum it is, so the bf16 matrix cores accumulate in fp32 exactly the terms of the fp32
// sum.  EXACT = false takes bf16 dY as it is.
#pragma once
#include "gemm_bf16.hip.h"

namespace paac {

template <class G, bool EXACT>
__global__ __launch_bounds__(256, 2) void conv1_wgrad_direct_kernel(const uint8_t* __restrict__ x, const void* __restrict__ dy_,
                                                                    float* __restrict__ pw, float* __restrict__ pb, int ns, float scale) {
    static_assert(G::CIN == 4 && G::H == 84 && G::W == 84 && G::KS == 8 && G::ST == 4 && G::COUT <= 32 && G::HO == 20 && G::WO == 20, "first layer");
    constexpr int SAMPLE = G::CIN * G::H * G::W, PLANE = G::H * G::W;
    constexpr int BR = 5, NB = G::HO / BR, IR = 4 * BR + 4;       // output rows per band, bands per sample, image rows per band
    constexpr int PW = 24;                                        // elements per phase row: x/4 = 0..20, zero beyond
    constexpr int COPY = 4 * IR * 4 * PW;                         // one de-interleaved band: [(c, y)][phase][PW]
    constexpr int NPART = EXACT ? 3 : 1, SP = 136;                // dY parts; slot pitch (128 slots + 8: conflict-free 16-byte reads)
    constexpr int IMG_ITEMS = 4 * IR * 6, IMG_IT = (IMG_ITEMS + 255) / 256;     // (c, y, quad of x/4) per band
    constexpr int QUADS = BR * 5;                                 // quads of positions per band
    // dY arrives as 16-byte loads (CPT channels of one position); a thread owns one quad of positions of one
    // channel group.  (One element per load, a thread per channel, was 64 of the 88 loads a wave issued per
    // band, and the rate at which a compute unit accepts loads bounded the kernel.)
    constexpr int CPT = EXACT ? 4 : 8, CGS = G::COUT / CPT, DY_UNITS = QUADS * CGS;
    static_assert(G::COUT % CPT == 0 && DY_UNITS <= 256, "one unit per thread");
    __shared__ __attribute__((aligned(16))) bf16_t img[2 * COPY];
    __shared__ __attribute__((aligned(16))) bf16_t dyt[NPART * 32 * SP];
    __shared__ float dbs[G::COUT * QUADS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int items = ns * NB;
    const int dcg = tid % CGS, dqd = tid / CGS;                   // this thread's channel group and quad of dY
    const bool dy_unit = tid < DY_UNITS;

    // raw data of the next item, in registers during the MFMA phase of the current one
    uint4 iw[IMG_IT]; uint32_t inx[IMG_IT];
    u32x4 dyr[4];
    auto prefetch = [&](int item) __attribute__((always_inline)) {
        const int s = item / NB, b = item % NB;
        const uint8_t* base = x + (size_t)s * SAMPLE + (size_t)(b * BR * G::ST) * G::W;
#pragma unroll
        for (int j = 0; j < IMG_IT; ++j) {
            const int ii = min(tid + j * 256, IMG_ITEMS - 1);     // clamped: a valid address, not stored
            const int c = ii / (IR * 6), y = (ii % (IR * 6)) / 6, q = ii % 6;
            const uint8_t* row = base + (size_t)c * PLANE + y * G::W;
            if (q < 5) {
                iw[j] = *reinterpret_cast<const uint4*>(row + 16 * q);           // x = 16 q .. 16 q + 15
                inx[j] = *reinterpret_cast<const uint32_t*>(row + 16 * q + 16);  // the next four (q = 4: x = 80 .. 83)
            } else {
                iw[j] = make_uint4(*reinterpret_cast<const uint32_t*>(row + 80), 0u, 0u, 0u);
                inx[j] = 0u;
            }
        }
        const size_t r0 = (size_t)s * (G::HO * G::WO) + (size_t)b * (BR * G::WO);
        const int qd = min(dqd, QUADS - 1);                       // threads without a unit: a valid address, not stored
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const size_t at = (r0 + 4 * qd + e) * G::COUT + dcg * CPT;
            if constexpr (EXACT) dyr[e] = *reinterpret_cast<const u32x4*>(static_cast<const float*>(dy_) + at);
            else dyr[e] = *reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(dy_) + at);
        }
    };
    auto pack_hi = [](float a, float b) __attribute__((always_inline)) {   // two fp32 with zero low halves -> two bf16 (exact: one packed conversion)
        return pack2(a, b);
    };

    int item = blockIdx.x;
    if (item >= items) return;
    prefetch(item);
    for (int i = tid; i < NPART * 32 * SP / 8; i += 256) reinterpret_cast<uint4*>(dyt)[i] = zero_u4();   // pad slots and channels stay zero

    f32x16 acc[2];
#pragma unroll
    for (int q = 0; q < 16; ++q) { acc[0][q] = 0.f; acc[1][q] = 0.f; }
    float db[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) db[c] = 0.f;

    // MFMA row m of a block of 32 k-values: m = (kx / 4) * 16 + ky_l * 4 + kx % 4 (sixteen lanes then read
    // sixteen different bank groups of one copy)
    const int m = lane & 31, half = lane >> 5;
    const int a_row = (m >> 4) * COPY + (((m >> 2) & 3) * 4 + (m & 3)) * PW;

    for (; item < items; item += gridDim.x) {
        __syncthreads();                                          // the previous item's fragments have been read
#pragma unroll
        for (int j = 0; j < IMG_IT; ++j) {
            const int ii = tid + j * 256;
            if (ii < IMG_ITEMS) {
                const int c = ii / (IR * 6), y = (ii % (IR * 6)) / 6, q = ii % 6;
                const uint32_t w[5] = {iw[j].x, iw[j].y, iw[j].z, iw[j].w, inx[j]};
                bf16_t* dst = img + ((c * IR + y) * 4) * PW + 4 * q;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    float f[5];
#pragma unroll
                    for (int e = 0; e < 5; ++e) f[e] = (float)((w[e] >> (8 * p)) & 255u);     // exact in bf16
                    *reinterpret_cast<uint2*>(dst + p * PW) = make_uint2(pack_hi(f[0], f[1]), pack_hi(f[2], f[3]));
                    *reinterpret_cast<uint2*>(dst + COPY + p * PW) = make_uint2(pack_hi(f[1], f[2]), pack_hi(f[3], f[4]));
                }
            }
        }
        if (dy_unit) {
            const int slot = (dqd / 5) * 24 + (dqd % 5) * 4;
#pragma unroll
            for (int c = 0; c < CPT; ++c) {                       // channel c of the group: its four positions as one 8-byte word per part
                bf16_t* at = dyt + (dcg * CPT + c) * SP + slot;
                if constexpr (EXACT) {
                    float v[4] = {__uint_as_float(dyr[0][c]), __uint_as_float(dyr[1][c]), __uint_as_float(dyr[2][c]), __uint_as_float(dyr[3][c])};
                    db[c] += (v[0] + v[1]) + (v[2] + v[3]);
#pragma unroll
                    for (int part = 0; part < NPART; ++part) {
                        float h[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            h[e] = __uint_as_float(__float_as_uint(v[e]) & 0xffff0000u);
                            v[e] -= h[e];                           // exact residual: the next part is cut from it
                        }
                        *reinterpret_cast<uint2*>(at + part * 32 * SP) = make_uint2(pack_hi(h[0], h[1]), pack_hi(h[2], h[3]));
                    }
                } else {
                    const unsigned sel = (c & 1) ? 0x07060302u : 0x05040100u;
                    uint2 o;
                    o.x = __builtin_amdgcn_perm(dyr[1][c >> 1], dyr[0][c >> 1], sel);
                    o.y = __builtin_amdgcn_perm(dyr[3][c >> 1], dyr[2][c >> 1], sel);
                    db[c] = dot2_ones(o.y, dot2_ones(o.x, db[c]));
                    *reinterpret_cast<uint2*>(at) = o;
                }
            }
        }
        __syncthreads();
        if (item + (int)gridDim.x < items) prefetch(item + gridDim.x);
        // the fragments of step t + 1 are read before the MFMAs of step t are issued
        u32x4 fa[2][2], fb[2][NPART];
        auto read_frags = [&](int t, int sl) __attribute__((always_inline)) {
            const int gi = min(2 * t + half, 14);                 // group 15 is all zero in dY: any valid image address
            const int oy = gi / 3, g = gi % 3;
            const bf16_t* ap = img + a_row + ((wave * IR + oy * G::ST) * 4) * PW + g * 8;
            fa[sl][0] = *reinterpret_cast<const u32x4*>(ap);                  // ky = ky_l
            fa[sl][1] = *reinterpret_cast<const u32x4*>(ap + 4 * 4 * PW);     // ky = 4 + ky_l
#pragma unroll
            for (int part = 0; part < NPART; ++part)
                fb[sl][part] = *reinterpret_cast<const u32x4*>(dyt + (part * 32 + m) * SP + t * 16 + half * 8);
        };
        read_frags(0, 0);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (t + 1 < 8) read_frags(t + 1, (t + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int part = NPART - 1; part >= 0; --part) {
                const bf16x8 bfr = __builtin_bit_cast(bf16x8, fb[t & 1][part]);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[t & 1][0]), bfr, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[t & 1][1]), bfr, acc[1], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // one partial per workgroup: dW[k][co] with k = c * 64 + ky * 8 + kx, c = wave
    float* out = pw + (size_t)blockIdx.x * (G::KK * G::COUT);
    if (m < G::COUT) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int r = Mma<32>::row(q, lane);
                const int kx = (r >> 4) * 4 + (r & 3), ky = blk * 4 + ((r >> 2) & 3);
                out[(wave * 64 + ky * 8 + kx) * G::COUT + m] = acc[blk][q] * scale;
            }
    }
    if (dy_unit) {
#pragma unroll
        for (int c = 0; c < CPT; ++c) dbs[(dcg * CPT + c) * QUADS + dqd] = db[c];
    }
    __syncthreads();
    if (tid < G::COUT) {
        float sdb = 0.f;
#pragma unroll
        for (int j = 0; j < QUADS; ++j) sdb += dbs[tid * QUADS + j];
        pb[(size_t)blockIdx.x * G::COUT + tid] = sdb;
    }
}

// n_wgs partials are written: pw [n_wgs][256][COUT], pb [n_wgs][COUT]; 1 <= n_wgs <= 4 ns.
template <class G, bool EXACT>
inline hipError_t launch_conv1_wgrad_direct(hipStream_t s, const uint8_t* x, const void* dy, float* pw, float* pb, int ns, int n_wgs) {
    if (ns <= 0 || n_wgs < 1 || n_wgs > ns * (G::HO / 5)) return hipErrorInvalidValue;
    launch_k((conv1_wgrad_direct_kernel<G, EXACT>), dim3(n_wgs), dim3(256), s, x, dy, pw, pb, ns, 1.0f / 255.0f);
    return hipGetLastError();
}

}  // namespace paac
