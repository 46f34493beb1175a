// Weight gradient of the second and third convolution with bf16 operands, one sample at a time from LDS.
//
//   dW[(ky,kx,ci)][co] = sum over samples and output positions (oy,ox) of X[ST oy + ky][ST ox + kx][ci] * dY[oy][ox][co]
//
// The reduction runs over output positions, and an MFMA lane must hold eight consecutive reduction
// indices of its row or column: both operands are position-major in memory, so both are transposed on
// their way into LDS.  As a tiled GEMM the im2col operand is gathered from global memory again for
// every tap (and the dY tile for every block of taps): 2.4 to 4 times the algorithmic bytes, and the
// compute units' L1 fill rate bounds the kernel.  Here a workgroup reads a sample once.
//
// Reduction index = (oy, slot t of 16): one 16-deep MFMA step per output row.
//   X^T  [ci][row = (y, parity of x)][16]   element e of a row is x = ST e + parity      (ST = 2)
//        [ci][y][16]                        element e is x = e                           (ST = 1)
//   dY^T [shift s][co][oy][16]              slot t holds ox = t - s, zero outside the map
// For tap (ky,kx) the input element that meets ox is e = ox + s with s = kx / 2 (ST = 2) or kx (ST = 1):
// with the dY copy shifted by s, slot t meets element e = t, so every fragment is an aligned 16-byte
// read: A = X^T[ci][row(ST oy + ky, kx)][8 half ..], B = dY^T[s][co][oy][8 half ..].  Channel and
// column pitches are odd multiples of 16 bytes (32 lanes read 32 different rows).
// The transposition: a thread takes four positions (elements e .. e+3, or slots t .. t+3) of eight
// channels (four 16-byte loads), transposes the 4 x 8 block in registers with byte permutes and writes
// eight 8-byte LDS words.  Waves own the MFMA row blocks (tap, 32-channel group) round robin and both
// 32-wide column blocks of each; a workgroup walks over samples and writes one partial dW and db.
#pragma once
#include "gemm_bf16.hip.h"

namespace paac {

template <class G> struct ConvWgradDirectShape {
    static constexpr int CIN = G::CIN, COUT = G::COUT, KS = G::KS, ST = G::ST;
    static_assert((ST == 1 || ST == 2) && CIN % 32 == 0 && COUT == 64, "layer shape");
    static constexpr int NPAR = ST, EPR = (G::W + NPAR - 1) / NPAR;       // parity planes, elements per transposed row
    static_assert(EPR <= 12 && G::WO + (ST == 2 ? 1 : KS - 1) <= 12, "three groups of four cover a row");
    static constexpr int XROWS = G::H * NPAR, CP = XROWS * 16 + 8;        // channel pitch (elements)
    static constexpr int NS = ST == 2 ? 2 : KS;                           // shifted copies of dY^T
    static constexpr int DP = G::HO * 16 + 8;                             // column pitch of dY^T
    static_assert((CP / 8) % 2 == 1 && (DP / 8) % 2 == 1, "pitches are odd multiples of 16 bytes");
    static constexpr int XT = CIN * CP, DYT = NS * COUT * DP;
    static constexpr int CF = CIN / 32, MF = KS * KS * CF, MPW = (MF + 3) / 4;      // MFMA row blocks, per wave
    static constexpr int XU = XROWS * (CIN / 8) * 3, DU = G::HO * (COUT / 8) * NS * 3;    // transposition units
    static constexpr int XIT = (XU + 255) / 256, DIT = (DU + 255) / 256, UIT = XIT + DIT;  // rounds of 256: first X, then dY
    // two images where they fit: a sample is then transposed while the previous one is multiplied
    static constexpr bool DB = 2 * (XT + DYT) * 2 + 4 * COUT * 4 <= 160 * 1024;
    static constexpr int IMG = XT + DYT;
    static constexpr int LDS_BYTES = (DB ? 2 : 1) * IMG * 2 + 4 * COUT * 4;
    static_assert(LDS_BYTES <= 160 * 1024, "fits the LDS of a compute unit");
};

template <class G>
__global__ __launch_bounds__(256, 1) void conv_wgrad_direct_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                                   float* __restrict__ pw, float* __restrict__ pb, int ns) {
    typedef ConvWgradDirectShape<G> S;
    constexpr int CIN = S::CIN, COUT = S::COUT, KS = S::KS, ST = S::ST, NPAR = S::NPAR, CP = S::CP, NS = S::NS, DP = S::DP;
    constexpr int CF = S::CF, MF = S::MF, MPW = S::MPW, XU = S::XU, DU = S::DU, XIT = S::XIT, UIT = S::UIT;
    constexpr int IN_POS = G::H * G::W, ROWS = G::HO * G::WO;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    bf16_t* const xt = reinterpret_cast<bf16_t*>(lds_raw);
    bf16_t* const dyt = xt + S::XT;
    float* const dbs = reinterpret_cast<float*>(xt + (S::DB ? 2 : 1) * S::IMG);          // [4 waves][COUT]
    constexpr bool DB = S::DB;
    constexpr int IMG = S::IMG;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 31, half = lane >> 5;

    // ---- this thread's transposition units: source offsets (elements within a sample, -1 = zero) and LDS target
    // (round i holds X units for i < XIT and dY units after that, so the operand of a round is a constant)
    int src[UIT][4], dst[UIT];
#pragma unroll
    for (int i = 0; i < UIT; ++i) {
        const int u = i < XIT ? tid + i * 256 : XU + tid + (i - XIT) * 256;
        dst[i] = -1;
#pragma unroll
        for (int q = 0; q < 4; ++q) src[i][q] = -1;
        if (i < XIT && u < XU) {
            const int g = u % 3, cg = (u / 3) % (CIN / 8), row = u / (3 * (CIN / 8));
            const int y = row / NPAR, par = row % NPAR;
            dst[i] = (cg * 8) * CP + row * 16 + g * 4;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int xx = (g * 4 + q) * NPAR + par;
                if (xx < G::W) src[i][q] = (y * G::W + xx) * CIN + cg * 8;
            }
        } else if (i >= XIT && u < XU + DU) {
            const int v = u - XU;
            const int g = v % 3, s = (v / 3) % NS, cg = (v / (3 * NS)) % (COUT / 8), oy = v / (3 * NS * (COUT / 8));
            dst[i] = S::XT + (s * COUT + cg * 8) * DP + oy * 16 + g * 4;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ox = g * 4 + q - s;
                if (ox >= 0 && ox < G::WO) src[i][q] = (oy * G::WO + ox) * COUT + cg * 8;
            }
        }
    }
    // Two register sets: the sample after next is requested as soon as this one's registers are free, so
    // a request has two whole samples' time to arrive (with one workgroup per compute unit nothing else
    // covers the latency; one sample ahead it was waited for, 1.5 us per sample).
    u32x4 raw[2][UIT][4];
    auto prefetch = [&](int smp, auto SET) __attribute__((always_inline)) {
        constexpr int set = decltype(SET)::value;
        const bf16_t* xs = x + (size_t)smp * (IN_POS * CIN);
        const bf16_t* ds = dy + (size_t)smp * (ROWS * COUT);
#pragma unroll
        for (int i = 0; i < UIT; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                raw[set][i][q] = *reinterpret_cast<const u32x4*>((i >= XIT ? ds : xs) + max(src[i][q], 0));     // clamped: masked below
    };
    int smp = blockIdx.x;
    if (smp >= ns) return;
    prefetch(smp, std::integral_constant<int, 0>());
    if (smp + (int)gridDim.x < ns) prefetch(smp + gridDim.x, std::integral_constant<int, 1>());
    // everything that no unit writes (row padding, slots outside the map) stays zero
    for (int i = tid; i < (DB ? 2 : 1) * IMG / 8; i += 256) reinterpret_cast<uint4*>(lds_raw)[i] = zero_u4();

    f32x16 acc[MPW][2];
#pragma unroll
    for (int i = 0; i < MPW; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) { acc[i][0][q] = 0.f; acc[i][1][q] = 0.f; }
    float db[2] = {0.f, 0.f};

    // one copy of the MFMA phase per wave keeps taps, shifts and accumulator indices constants
    auto per_wave = [&](auto&& fn) __attribute__((always_inline)) {
        if (wave == 0) fn(std::integral_constant<int, 0>());
        if (wave == 1) fn(std::integral_constant<int, 1>());
        if (wave == 2) fn(std::integral_constant<int, 2>());
        if (wave == 3) fn(std::integral_constant<int, 3>());
    };

    // round i of the transposition of the sample in register set SET, into image `buf`
    auto transpose_round = [&](auto RI, auto SET, int buf) __attribute__((always_inline)) {
        constexpr int i = decltype(RI)::value, set = decltype(SET)::value;
        if (dst[i] >= 0) {
            uint32_t w[4][4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool ok = src[i][q] >= 0;
                w[q][0] = ok ? raw[set][i][q].x : 0u; w[q][1] = ok ? raw[set][i][q].y : 0u;
                w[q][2] = ok ? raw[set][i][q].z : 0u; w[q][3] = ok ? raw[set][i][q].w : 0u;
            }
            bf16_t* d = xt + buf * IMG + dst[i];       // dY^T follows X^T
            constexpr int pitch_i = i >= XIT ? DP : CP;
#pragma unroll
            for (int j = 0; j < 8; ++j) {              // channel j of the eight: positions 0..3 as one 8-byte word
                const unsigned sel = (j & 1) ? 0x07060302u : 0x05040100u;
                uint2 o;
                o.x = __builtin_amdgcn_perm(w[1][j >> 1], w[0][j >> 1], sel);
                o.y = __builtin_amdgcn_perm(w[3][j >> 1], w[2][j >> 1], sel);
                *reinterpret_cast<uint2*>(d + j * pitch_i) = o;
            }
        }
    };
    auto transpose_all = [&](auto SET, int buf) __attribute__((always_inline)) {
        [&]<int... I>(std::integer_sequence<int, I...>) {
            (transpose_round(std::integral_constant<int, I>(), SET, buf), ...);
        }(std::make_integer_sequence<int, UIT>());
    };
    // MFMA phase on image `buf`; between(oy) runs after the MFMAs of output row oy have been issued
    auto mfma_phase = [&](int buf, auto&& between) __attribute__((always_inline)) {
        const bf16_t* const xb = xt + buf * IMG;
        const bf16_t* const db_ = xb + S::XT;
        per_wave([&](auto WV) __attribute__((always_inline)) {
            constexpr int wv = decltype(WV)::value;
            // fragments of output row oy + 1 are read before the MFMAs of row oy are issued
            u32x4 bq[2][NS][2], aq[2][MPW];
            auto read_frags = [&](auto OY, auto SLOT) __attribute__((always_inline)) {
                constexpr int oy = decltype(OY)::value, sl = decltype(SLOT)::value;
#pragma unroll
                for (int s = 0; s < NS; ++s)
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb)
                        bq[sl][s][cb] = *reinterpret_cast<const u32x4*>(db_ + (s * COUT + cb * 32 + m) * DP + oy * 16 + half * 8);
#pragma unroll
                for (int i = 0; i < MPW; ++i) {
                    const int mf = wv + 4 * i;
                    if (mf < MF) {
                        const int tap = mf / CF, cf = mf % CF, ky = tap / KS, kx = tap % KS;
                        const int par = ST == 2 ? (kx & 1) : 0;
                        aq[sl][i] = *reinterpret_cast<const u32x4*>(xb + (cf * 32 + m) * CP + ((ST * oy + ky) * NPAR + par) * 16 + half * 8);
                    }
                }
            };
            read_frags(std::integral_constant<int, 0>(), std::integral_constant<int, 0>());
            [&]<int... OY>(std::integer_sequence<int, OY...>) {
                ([&] {
                    constexpr int oy = OY, sl = OY & 1;
                    if constexpr (oy + 1 < G::HO) read_frags(std::integral_constant<int, oy + 1>(), std::integral_constant<int, sl ^ 1>());
                    __builtin_amdgcn_sched_barrier(0);
                    if (oy % 4 == wv) {                // bias gradient: the unshifted copy's slots, spread over the waves
#pragma unroll
                        for (int cb = 0; cb < 2; ++cb) {
                            const u32x4 v = bq[sl][0][cb];
                            db[cb] = dot2_ones(v.w, dot2_ones(v.z, dot2_ones(v.y, dot2_ones(v.x, db[cb]))));
                        }
                    }
#pragma unroll
                    for (int i = 0; i < MPW; ++i) {
                        const int mf = wv + 4 * i;
                        if (mf < MF) {
                            const int tap = mf / CF, kx = tap % KS;
                            const int s = ST == 2 ? kx >> 1 : kx;
                            const bf16x8 a = __builtin_bit_cast(bf16x8, aq[sl][i]);
                            acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, bq[sl][s][0]), acc[i][0], 0, 0, 0);
                            acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, bq[sl][s][1]), acc[i][1], 0, 0, 0);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    between(std::integral_constant<int, oy>());
                }(), ...);
            }(std::make_integer_sequence<int, G::HO>());
        });
    };
    const int g = gridDim.x;
    if constexpr (!DB) {
        auto one_sample = [&](auto SET) __attribute__((always_inline)) {
            __syncthreads();                           // the previous sample's fragments have been read (first pass: the zeros are written)
            transpose_all(SET, 0);
            if (smp + 2 * g < ns) prefetch(smp + 2 * g, SET);
            __syncthreads();
            mfma_phase(0, [](auto) {});
        };
        for (;;) {
            one_sample(std::integral_constant<int, 0>());
            smp += g;
            if (smp >= ns) break;
            one_sample(std::integral_constant<int, 1>());
            smp += g;
            if (smp >= ns) break;
        }
    } else {
        // Two images: while the waves multiply sample k from image k % 2, they transpose sample k + 1
        // (register set (k + 1) % 2) into the other image, a round after every few output rows, in the
        // shadow of the MFMAs; one barrier per sample.
        __syncthreads();                               // the zeros are written
        transpose_all(std::integral_constant<int, 0>(), 0);
        if (smp + 2 * g < ns) prefetch(smp + 2 * g, std::integral_constant<int, 0>());
        auto one_sample = [&](int buf, auto NEXT) __attribute__((always_inline)) {
            __syncthreads();                           // image `buf` is complete, the other one is no longer read
            const bool has_next = smp + g < ns;
            mfma_phase(buf, [&](auto OY) __attribute__((always_inline)) {
                constexpr int oy = decltype(OY)::value;
                [&]<int... I>(std::integer_sequence<int, I...>) {
                    ([&] {
                        if constexpr (I * G::HO / UIT == oy) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (has_next) transpose_round(std::integral_constant<int, I>(), NEXT, buf ^ 1);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }(), ...);
                }(std::make_integer_sequence<int, UIT>());
            });
            if (smp + 3 * g < ns) prefetch(smp + 3 * g, NEXT);
        };
        for (;;) {
            one_sample(0, std::integral_constant<int, 1>());
            smp += g;
            if (smp >= ns) break;
            one_sample(1, std::integral_constant<int, 0>());
            smp += g;
            if (smp >= ns) break;
        }
    }

    // ---- one partial per workgroup: dW[k = tap * CIN + ci][co], db[co]
    float* out = pw + (size_t)blockIdx.x * (G::KK * COUT);
    per_wave([&](auto WV) __attribute__((always_inline)) {
        constexpr int wv = decltype(WV)::value;
#pragma unroll
        for (int i = 0; i < MPW; ++i) {
            const int mf = wv + 4 * i;
            if (mf < MF) {
                const int tap = mf / CF, cf = mf % CF;
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        out[(size_t)(tap * CIN + cf * 32 + Mma<32>::row(q, lane)) * COUT + cb * 32 + m] = acc[i][cb][q];
            }
        }
    });
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const float t = db[cb] + __shfl_xor(db[cb], 32);
        if (half == 0) dbs[wave * COUT + cb * 32 + m] = t;
    }
    __syncthreads();
    if (tid < COUT) pb[(size_t)blockIdx.x * COUT + tid] = ((dbs[tid] + dbs[COUT + tid]) + dbs[2 * COUT + tid]) + dbs[3 * COUT + tid];
}

// n_wgs partials are written: pw [n_wgs][KK][COUT], pb [n_wgs][COUT]; 1 <= n_wgs <= ns.
template <class G>
inline hipError_t launch_conv_wgrad_direct(hipStream_t s, const bf16_t* x, const bf16_t* dy, float* pw, float* pb, int ns, int n_wgs) {
    if (ns <= 0 || n_wgs < 1 || n_wgs > ns) return hipErrorInvalidValue;
    constexpr int LDS = ConvWgradDirectShape<G>::LDS_BYTES;
    static bool ready = false;
    if (!ready) {                       // more LDS than a kernel gets by default
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_wgrad_direct_kernel<G>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        ready = true;
    }
    launch_k_lds((conv_wgrad_direct_kernel<G>), dim3(n_wgs), dim3(256), LDS, s, x, dy, pw, pb, ns);
    return hipGetLastError();
}

}  // namespace paac
