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
// A lane's eight reduction indices are one 16-byte LDS read; the two halves of a wave may read
// anywhere, so a 16-deep MFMA step is any two groups of eight positions.  The groups:
//   row part     the first eight output columns (seven exist in the third layer) of one output row;
//                a k-step is two output rows, oy = 2 kk + lane half
//   column part  (second layer: nine columns) the ninth column, its nine output rows in one group of 16
// so a sample is 4 k-steps (49 positions in 64 slots) or 6 (81 in 96); with one output row per step
// padded to 16 slots it was 7 and 9.
//   X^T  [shift s][ci][row][8]   element j of a row is x = ST (j + s) + parity; row = y (ST = 1) or (y, parity of x)
//                                tap kx reads shift s = kx (ST = 1) or kx / 2 and parity kx % 2, so that
//                                element j meets output column j: every fragment an aligned 16-byte read
//   dY^T [co][oy][8]             element j is ox = j, zero where no such output exists
//   X^C  [ci][tap][16]           element j is X[ST j + ky][ST 8 + kx]   (column part)
//   dY^C [co][16]                element j is dY[j][8]
// Rows past the map (the partner of the last output row when their number is odd, and the input rows
// its taps reach) are never written and stay zero.  Channel pitches are odd multiples of 16 bytes:
// the sixteen lanes that one cycle of a 16-byte read serves hit sixteen different bank groups.  Eight
// channels on, an odd pitch is 128 bytes on modulo the 256 of the banks, sixteen channels on it is
// back at 0: in X^T every second group of sixteen channels therefore starts 64 bytes later (a read's
// sixteen lanes are one such group, so nothing changes for them), and the transposition's 8-byte
// writes of four neighbouring channel groups land in four different quarters of the banks.
// The transposition: a thread takes four positions of eight channels (four 16-byte loads), transposes
// the 4 x 8 block in registers with byte permutes and writes eight 8-byte LDS words.  In the order of
// the units over the lanes, four neighbouring channel groups come first (64 contiguous bytes of a
// position: a wave's load touches 16 such segments; with one segment per lane the address pipeline took
// 2 400 cycles per sample to accept the loads), then half rows and rows (a write of the wave then meets
// sixteen lanes, which the LDS serves together, in sixteen different places: 8 cycles; without the
// 64-byte offsets 16, and with all eight channel groups of a position side by side 21).  dY^T and the
// column part keep plain pitches (there is no LDS left for theirs in the second layer, and they are
// a third of the writes).
// A workgroup is eight waves with two roles and two images: waves 4-7 request a sample's data two samples
// ahead, transpose it and write the image of sample k + 1 while waves 0-3 read the fragments of sample k
// and issue its MFMAs (the 32 x 32 output tiles (tap, 32-channel group) x (half of the output channels)
// dealt evenly to them); one barrier per sample.  With four waves doing everything in turn, one per SIMD,
// nothing covered a wave's own stalls (third layer 145 -> 112 us, second 240 -> 178 us at 20 480 samples).
// A workgroup walks over samples and writes one partial dW and db.
#pragma once
#include "gemm_bf16.hip.h"

namespace paac {

template <class G> struct ConvWgradDirectShape {
    static constexpr int CIN = G::CIN, COUT = G::COUT, KS = G::KS, ST = G::ST, TAPS = KS * KS;
    static_assert((ST == 1 || ST == 2) && CIN % 32 == 0 && COUT == 64, "layer shape");
    static constexpr int NPAR = ST;                                       // x-parity planes of the input
    static constexpr bool COLPART = G::WO > 8;
    static constexpr int COLS = COLPART ? 8 : G::WO;                      // output columns of the row part
    static_assert(G::WO <= 9 && G::HO <= 16, "at most one column beyond the row part, its rows in one 16-deep step");
    static constexpr int KROW = (G::HO + 1) / 2, KSTEPS = KROW + (COLPART ? 1 : 0);
    static constexpr int NSH = ST == 2 ? KS / 2 : KS;                     // shifted copies of X^T
    static constexpr int YR = ST * (2 * KROW - 1) + KS;                   // input rows the taps of the row part reach
    static constexpr int XROWS = YR * NPAR, DROWS = 2 * KROW;
    static constexpr int SKEW = 32;                                       // elements: odd groups of 16 channels of X^T start 64 bytes later
    static constexpr int CP = XROWS * 8 + SKEW + (XROWS % 2 ? 16 : 8);    // channel pitch of X^T (elements)
    static constexpr int DP = DROWS * 8 + 8;                              // column pitch of dY^T
    static constexpr int XCP = TAPS * 16 + 8, DCP = 24;                      // pitches of the column part
    static_assert((CP / 8) % 2 == 1 && (DP / 8) % 2 == 1 && (XCP / 8) % 2 == 1 && (DCP / 8) % 2 == 1, "pitches are odd multiples of 16 bytes");
    static constexpr int XT = NSH * CIN * CP, DYT = COUT * DP;
    static constexpr int XCT = COLPART ? CIN * XCP : 0, DCT = COLPART ? COUT * DCP : 0;
    static constexpr int IMG = XT + DYT + XCT + DCT;
    // transposition units (4 positions x 8 channels), in the order X^T, dY^T, X^C, dY^C
    static constexpr int XU = NSH * G::H * NPAR * 2 * (CIN / 8), DU = G::HO * 2 * (COUT / 8);
    static constexpr int CG4 = (G::HO + 3) / 4;                           // groups of four elements in a column
    static constexpr int XCU = COLPART ? TAPS * CG4 * (CIN / 8) : 0, DCU = COLPART ? CG4 * (COUT / 8) : 0;
    static constexpr int UNITS = XU + DU + XCU + DCU, UIT = (UNITS + 255) / 256;
    static constexpr int CF = CIN / 32, MF = TAPS * CF, TILES = MF * 2, TPW = TILES / 4;    // 32 x 32 output tiles, per wave
    static_assert(TILES % 4 == 0, "equal shares of the output tiles");
    static constexpr int NA = TPW / 2 + 1;                                // row blocks a wave's tiles touch, at most
    // two images: a sample is transposed while the previous one is multiplied
    static constexpr int LDS_BYTES = 2 * IMG * 2 + 4 * COUT * 4;
    static_assert(LDS_BYTES <= 160 * 1024, "fits the LDS of a compute unit");
};

template <class G>
__global__ __launch_bounds__(512, 1) void conv_wgrad_direct_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                                   float* __restrict__ pw, float* __restrict__ pb, int ns) {
    typedef ConvWgradDirectShape<G> S;
    constexpr int CIN = S::CIN, COUT = S::COUT, KS = S::KS, ST = S::ST, NPAR = S::NPAR, CP = S::CP, DP = S::DP, XCP = S::XCP, DCP = S::DCP;
    constexpr int CF = S::CF, TPW = S::TPW, NA = S::NA, UIT = S::UIT, KROW = S::KROW, KSTEPS = S::KSTEPS;
    constexpr int IN_POS = G::H * G::W, ROWS = G::HO * G::WO;
    constexpr int IMG = S::IMG;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    bf16_t* const img0 = reinterpret_cast<bf16_t*>(lds_raw);
    float* const dbs = reinterpret_cast<float*>(img0 + 2 * IMG);                        // [4 waves][COUT]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = gridDim.x;
    int smp = blockIdx.x;
    if (smp >= ns) return;
    // everything that no unit writes (rows past the map, elements past a column's end) stays zero
    for (int i = tid; i < 2 * IMG / 8; i += 512) reinterpret_cast<uint4*>(lds_raw)[i] = zero_u4();
    __syncthreads();

    if (wave >= 4) {
        // ================= waves 4-7: global memory -> registers -> transposed images =================
        const int lt = tid - 256;
        // this thread's transposition units: source offsets (elements within a sample of x or dy, -1 = zero),
        // LDS target of channel 0 of the eight, and the target's channel pitch
        int src[UIT][4], dst[UIT], pitch[UIT];
        bool from_dy[UIT];
#pragma unroll
        for (int i = 0; i < UIT; ++i) {
            int u = lt + i * 256;
            dst[i] = -1; pitch[i] = 0; from_dy[i] = false;
#pragma unroll
            for (int q = 0; q < 4; ++q) src[i][q] = -1;
            if (u < S::XU) {
                const int gq = (u / 4) % 2, row = (u / 8) % (G::H * NPAR), cg = u % 4 + 4 * ((u / (8 * G::H * NPAR)) % (CIN / 32)), sh = u / (2 * G::H * NPAR * (CIN / 8));
                const int y = row / NPAR, par = row % NPAR;
                dst[i] = (sh * CIN + cg * 8) * CP + ((cg >> 1) & 1) * S::SKEW + row * 8 + gq * 4; pitch[i] = CP;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int xx = ST * (gq * 4 + q + sh) + par;
                    if (xx < G::W) src[i][q] = (y * G::W + xx) * CIN + cg * 8;
                }
            } else if ((u -= S::XU) < S::DU) {
                const int gq = (u / 4) % 2, oy = (u / 8) % G::HO, cg = u % 4 + 4 * (u / (8 * G::HO));
                dst[i] = S::XT + (cg * 8) * DP + oy * 8 + gq * 4; pitch[i] = DP; from_dy[i] = true;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int ox = gq * 4 + q;
                    if (ox < S::COLS) src[i][q] = (oy * G::WO + ox) * COUT + cg * 8;
                }
            } else if ((u -= S::DU) < S::XCU) {
                const int gq = (u / 4) % S::CG4, cg = u % 4 + 4 * ((u / (4 * S::CG4)) % (CIN / 32)), tap = u / (S::CG4 * (CIN / 8));
                dst[i] = S::XT + S::DYT + (cg * 8) * XCP + tap * 16 + gq * 4; pitch[i] = XCP;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = gq * 4 + q;
                    if (j < G::HO) src[i][q] = ((ST * j + tap / KS) * G::W + ST * 8 + tap % KS) * CIN + cg * 8;
                }
            } else if ((u -= S::XCU) < S::DCU) {
                const int gq = (u / 4) % S::CG4, cg = u % 4 + 4 * (u / (4 * S::CG4));
                dst[i] = S::XT + S::DYT + S::XCT + (cg * 8) * DCP + gq * 4; pitch[i] = DCP; from_dy[i] = true;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = gq * 4 + q;
                    if (j < G::HO) src[i][q] = (j * G::WO + 8) * COUT + cg * 8;
                }
            }
        }
        // Two register sets: the sample after next is requested as soon as this one's registers are free,
        // so a request has two whole samples' time to arrive.
        u32x4 raw[2][UIT][4];
        auto prefetch = [&](int sm, auto SET) __attribute__((always_inline)) {
            constexpr int set = decltype(SET)::value;
            const bf16_t* xs = x + (size_t)sm * (IN_POS * CIN);
            const bf16_t* ds = dy + (size_t)sm * (ROWS * COUT);
#pragma unroll
            for (int i = 0; i < UIT; ++i) {
                const bf16_t* from = from_dy[i] ? ds : xs;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    raw[set][i][q] = *reinterpret_cast<const u32x4*>(from + max(src[i][q], 0));     // clamped: masked below
            }
        };
        auto transpose_all = [&](auto SET, int buf) __attribute__((always_inline)) {
            constexpr int set = decltype(SET)::value;
#pragma unroll
            for (int i = 0; i < UIT; ++i)
                if (dst[i] >= 0) {
                    uint32_t w[4][4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const bool ok = src[i][q] >= 0;
                        w[q][0] = ok ? raw[set][i][q].x : 0u; w[q][1] = ok ? raw[set][i][q].y : 0u;
                        w[q][2] = ok ? raw[set][i][q].z : 0u; w[q][3] = ok ? raw[set][i][q].w : 0u;
                    }
                    bf16_t* d = img0 + buf * IMG + dst[i];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {      // channel j of the eight: positions 0..3 as one 8-byte word
                        const unsigned sel = (j & 1) ? 0x07060302u : 0x05040100u;
                        uint2 o;
                        o.x = __builtin_amdgcn_perm(w[1][j >> 1], w[0][j >> 1], sel);
                        o.y = __builtin_amdgcn_perm(w[3][j >> 1], w[2][j >> 1], sel);
                        *reinterpret_cast<uint2*>(d + j * pitch[i]) = o;
                    }
                }
        };
        prefetch(smp, std::integral_constant<int, 0>());
        if (smp + g < ns) prefetch(smp + g, std::integral_constant<int, 1>());
        transpose_all(std::integral_constant<int, 0>(), 0);
        if (smp + 2 * g < ns) prefetch(smp + 2 * g, std::integral_constant<int, 0>());
        __syncthreads();                               // image 0 holds the first sample
        // while the other waves multiply sample k from image k % 2: sample k + 1 into the other image
        auto one_sample = [&](int buf, auto NEXT) __attribute__((always_inline)) {
            if (smp + g < ns) {
                transpose_all(NEXT, buf ^ 1);
                if (smp + 3 * g < ns) prefetch(smp + 3 * g, NEXT);
            }
            __syncthreads();                           // image buf ^ 1 is complete, image buf has been read
        };
        for (;;) {
            one_sample(0, std::integral_constant<int, 1>());
            smp += g;
            if (smp >= ns) break;
            one_sample(1, std::integral_constant<int, 0>());
            smp += g;
            if (smp >= ns) break;
        }
    } else {
        // ================= waves 0-3: fragments from the images, MFMA =================
        const int m = lane & 31, half = lane >> 5;
        f32x16 acc[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][q] = 0.f;
        float db[2] = {0.f, 0.f};
        // one copy of the MFMA phase per wave keeps taps, shifts and accumulator indices constants
        auto per_wave = [&](auto&& fn) __attribute__((always_inline)) {
            if (wave == 0) fn(std::integral_constant<int, 0>());
            if (wave == 1) fn(std::integral_constant<int, 1>());
            if (wave == 2) fn(std::integral_constant<int, 2>());
            if (wave == 3) fn(std::integral_constant<int, 3>());
        };
        // this lane's part of every fragment address (elements)
        const int la = m * CP + ((m >> 4) & 1) * S::SKEW + half * (ST == 2 ? 32 : 8);     // X^T: the second output row of a k-step is ST input rows on
        const int lb = S::XT + m * DP + half * 8;
        const int lac = S::XT + S::DYT + m * XCP + half * 8;
        const int lbc = S::XT + S::DYT + S::XCT + m * DCP + half * 8;
        auto mfma_phase = [&](int buf) __attribute__((always_inline)) {
            const bf16_t* const ib = img0 + buf * IMG;
            per_wave([&](auto WV) __attribute__((always_inline)) {
                constexpr int wv = decltype(WV)::value;
                constexpr int T0 = wv * TPW, MF0 = T0 / 2;     // this wave's tiles t = T0 + i: row block t / 2, column block t % 2
                // fragments of k-step kk + 1 are read before the MFMAs of kk are issued
                u32x4 bq[2][2], aq[2][NA];
                auto read_frags = [&](auto KK, auto SLOT) __attribute__((always_inline)) {
                    constexpr int kk = decltype(KK)::value, sl = decltype(SLOT)::value;
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb)
                        bq[sl][cb] = *reinterpret_cast<const u32x4*>(ib + (kk < KROW ? lb + cb * 32 * DP + 2 * kk * 8 : lbc + cb * 32 * DCP));
#pragma unroll
                    for (int a = 0; a < NA; ++a) {
                        const int mf = MF0 + a;
                        if (2 * mf < T0 + TPW) {
                            const int tap = mf / CF, cf = mf % CF, ky = tap / KS, kx = tap % KS;
                            const int sh = ST == 2 ? kx >> 1 : kx, par = ST == 2 ? kx & 1 : 0;
                            const int row = (ST * 2 * kk + ky) * NPAR + par;
                            aq[sl][a] = *reinterpret_cast<const u32x4*>(ib + (kk < KROW ? la + (sh * CIN + cf * 32) * CP + row * 8
                                                                                        : lac + cf * 32 * XCP + tap * 16));
                        }
                    }
                };
                read_frags(std::integral_constant<int, 0>(), std::integral_constant<int, 0>());
                [&]<int... KK>(std::integer_sequence<int, KK...>) {
                    ([&] {
                        constexpr int kk = KK, sl = KK & 1;
                        if constexpr (kk + 1 < KSTEPS) read_frags(std::integral_constant<int, kk + 1>(), std::integral_constant<int, sl ^ 1>());
                        __builtin_amdgcn_sched_barrier(0);
                        if (kk % 4 == wv) {            // bias gradient: every element of dY is in exactly one k-step's fragments
#pragma unroll
                            for (int cb = 0; cb < 2; ++cb) {
                                const u32x4 v = bq[sl][cb];
                                db[cb] = dot2_ones(v.w, dot2_ones(v.z, dot2_ones(v.y, dot2_ones(v.x, db[cb]))));
                            }
                        }
#pragma unroll
                        for (int i = 0; i < TPW; ++i) {
                            const int t = T0 + i;
                            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aq[sl][t / 2 - MF0]),
                                                                             __builtin_bit_cast(bf16x8, bq[sl][t % 2]), acc[i], 0, 0, 0);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }(), ...);
                }(std::make_integer_sequence<int, KSTEPS>());
            });
        };
        __syncthreads();                               // image 0 holds the first sample
        for (;;) {
            mfma_phase(0);
            __syncthreads();
            smp += g;
            if (smp >= ns) break;
            mfma_phase(1);
            __syncthreads();
            smp += g;
            if (smp >= ns) break;
        }
        // ---- one partial per workgroup: dW[k = tap * CIN + ci][co]
        float* out = pw + (size_t)blockIdx.x * (G::KK * COUT);
        per_wave([&](auto WV) __attribute__((always_inline)) {
            constexpr int wv = decltype(WV)::value;
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int t = wv * TPW + i, mf = t / 2, cb = t % 2;
                const int tap = mf / CF, cf = mf % CF;
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    out[(size_t)(tap * CIN + cf * 32 + Mma<32>::row(q, lane)) * COUT + cb * 32 + m] = acc[i][q];
            }
        });
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const float t = db[cb] + __shfl_xor(db[cb], 32);
            if (half == 0) dbs[wave * COUT + cb * 32 + m] = t;
        }
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
    launch_k_lds((conv_wgrad_direct_kernel<G>), dim3(n_wgs), dim3(512), LDS, s, x, dy, pw, pb, ns);
    return hipGetLastError();
}

}  // namespace paac
