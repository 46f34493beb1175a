// Tiled GEMM core with bf16 operands on v_mfma_f32_32x32x16_bf16 (fp32 accumulation), for the
// configurations that run the conv/fc contractions in bf16 (activations and weight copies in bf16,
// fp32 master weights, fp32 heads / losses / optimiser).
//
//   C[m][n] = sum_k A(m,k) * B(k,n)
//
// The MFMA wants, per lane, eight consecutive k of one row (A) or column (B).  Two staging modes:
//   RowK (forward, data gradient): both operands are contiguous along k in memory; a tile is
//        kept in LDS as [row][BK] and a lane reads its eight k with one 16-byte LDS load.
//   KRow (weight gradient): the reduction runs over output positions, both operands are
//        contiguous along m / n; a tile is kept as [k][cols] and a lane gathers its eight k with
//        eight 2-byte LDS loads (a transposition done by addressing, no data movement).
// Global loads are 16 bytes (8 bf16; 8 bytes for the uint8 first layer), branch free and clamped,
// S register stages ahead; conversion and zeroing happen when the registers are stored to LDS.
#pragma once
#include "gemm_core.hip.h"

namespace paac {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ bf16_t f2bf(float f) { __bf16 b = (__bf16)f; return __builtin_bit_cast(unsigned short, b); }
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float((unsigned)h << 16); }
__device__ __forceinline__ unsigned pack2(float lo, float hi) { return (unsigned)f2bf(lo) | ((unsigned)f2bf(hi) << 16); }
__device__ __forceinline__ uint4 zero_u4() { return make_uint4(0u, 0u, 0u, 0u); }
__device__ __forceinline__ uint4 keep_if_u4(bool ok, uint4 v) {
    return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
}
// eight bytes -> eight bf16 holding the byte values 0..255 exactly (8 significand bits suffice);
// the 1/255 of the input scaling is applied to the fp32 accumulators in the epilogue instead, so the
// first layer's input carries no rounding error at all
__device__ __forceinline__ uint4 u8x8_to_bf16(uint2 w) {
    auto cv = [&](unsigned x, int sh) { return (float)((x >> sh) & 255u); };
    return make_uint4(pack2(cv(w.x, 0), cv(w.x, 8)), pack2(cv(w.x, 16), cv(w.x, 24)),
                      pack2(cv(w.y, 0), cv(w.y, 8)), pack2(cv(w.y, 16), cv(w.y, 24)));
}

template <int BM_, int BN_, int BK_, int WM_, int WN_, int STAGES_ = 3>
struct TileB {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, STAGES = STAGES_;
    static constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(TM * WM * 32 == BM && TN * WN * 32 == BN, "tile must be whole 32x32 fragments");
    static_assert(BK % 16 == 0, "BK must be a multiple of the MFMA depth");
};

// Operand functor interface (8-wide):
//   static constexpr bool kContig;      true: RowK operand (fixed = row, var = k, multiple of 8)
//                                       false: KRow operand (fixed = first of 8 columns, var = k)
//   typedef Raw; Raw load(fixed, var, pred, ok&);  static uint4 finish(Raw, ok)  -> 8 bf16
template <class T, class AL, class BL, class EP>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const AL al, const BL bl, const EP ep, int M, int N, int K,
                                                        int k_per_split, int m_tiles) {
    static_assert(AL::kContig == BL::kContig, "both operands use the same staging mode");
    constexpr bool ROWK = AL::kContig;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, TM = T::TM, TN = T::TN, S = T::STAGES;
    // leading dimensions in bf16 elements: 16 bytes of padding keep the 16-byte rows aligned and
    // rotate the banks from row to row
    constexpr int LDA = ROWK ? BK + 8 : BM + 8;
    constexpr int LDB = ROWK ? BK + 8 : BN + 8;
    constexpr int A_BUF = (ROWK ? BM : BK) * LDA, B_BUF = (ROWK ? BN : BK) * LDB;
    constexpr int A_U = BM * BK / 8, B_U = BN * BK / 8;          // 16-byte units per tile
    constexpr int A_IT = (A_U + 255) / 256, B_IT = (B_U + 255) / 256;
    static_assert(A_IT + B_IT <= 16, "ok-bit mask");

    __shared__ __attribute__((aligned(16))) bf16_t smem[2 * A_BUF + 2 * B_BUF];
    bf16_t* const As = smem;
    bf16_t* const Bs = smem + 2 * A_BUF;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % T::WM, wn = wave / T::WM;
    const int mt = blockIdx.x % m_tiles, nt = blockIdx.x / m_tiles;
    const int z = blockIdx.y;
    const int m0 = mt * BM, n0 = nt * BN;
    const int k_begin = k_per_split > 0 ? z * k_per_split : 0;
    const int k_end = k_per_split > 0 ? min(K, k_begin + k_per_split) : K;
    const int nk = (k_end - k_begin + BK - 1) / BK;

    typename AL::Fixed afix[A_IT];
    typename BL::Fixed bfix[B_IT];
    int a_var[A_IT], a_lds[A_IT], b_var[B_IT], b_lds[B_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        const int f = tid + i * 256;
        if (ROWK) {
            const int kq = f % (BK / 8), row = f / (BK / 8);
            afix[i] = al.prep(m0 + row, z); a_var[i] = kq * 8; a_lds[i] = row * LDA + kq * 8;
        } else {
            const int cq = f % (BM / 8), k = f / (BM / 8);
            afix[i] = al.prep(m0 + cq * 8, z); a_var[i] = k; a_lds[i] = k * LDA + cq * 8;
        }
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
        const int f = tid + i * 256;
        if (ROWK) {
            const int kq = f % (BK / 8), row = f / (BK / 8);
            bfix[i] = bl.prep(n0 + row, z); b_var[i] = kq * 8; b_lds[i] = row * LDB + kq * 8;
        } else {
            const int cq = f % (BN / 8), k = f / (BN / 8);
            bfix[i] = bl.prep(n0 + cq * 8, z); b_var[i] = k; b_lds[i] = k * LDB + cq * 8;
        }
    }

    typename AL::Raw areg[S][A_IT];
    typename BL::Raw breg[S][B_IT];
    unsigned okbits[S];
    auto gload = [&](int kt, auto stage) {
        constexpr int G = decltype(stage)::value;
        const int kb = k_begin + kt * BK;
        unsigned bits = 0;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int kk = kb + a_var[i];
            bool ok;
            areg[G][i] = al.load(afix[i], kk, (A_U % 256 == 0 || tid + i * 256 < A_U) && kk < k_end, ok);
            bits |= ok ? (1u << i) : 0u;
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const int kk = kb + b_var[i];
            bool ok;
            breg[G][i] = bl.load(bfix[i], kk, (B_U % 256 == 0 || tid + i * 256 < B_U) && kk < k_end, ok);
            bits |= ok ? (1u << (16 + i)) : 0u;
        }
        okbits[G] = bits;
    };
    auto lstore = [&](auto stage, int buf) {
        constexpr int G = decltype(stage)::value;
#pragma unroll
        for (int i = 0; i < A_IT; ++i)
            if (tid + i * 256 < A_U)
                *reinterpret_cast<uint4*>(As + buf * A_BUF + a_lds[i]) = AL::finish(areg[G][i], (okbits[G] >> i) & 1u);
#pragma unroll
        for (int i = 0; i < B_IT; ++i)
            if (tid + i * 256 < B_U)
                *reinterpret_cast<uint4*>(Bs + buf * B_BUF + b_lds[i]) = BL::finish(breg[G][i], (okbits[G] >> (16 + i)) & 1u);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    float colsum = 0.f;

    const int fidx = lane & 31, kg = lane >> 5;
    auto compute = [&](int buf) {
        const bf16_t* as = As + buf * A_BUF;
        const bf16_t* bs = Bs + buf * B_BUF;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 a[TM], b[TN];
            if constexpr (ROWK) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    a[i] = *reinterpret_cast<const bf16x8*>(as + (wm * TM * 32 + i * 32 + fidx) * LDA + ks * 16 + kg * 8);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    b[j] = *reinterpret_cast<const bf16x8*>(bs + (wn * TN * 32 + j * 32 + fidx) * LDB + ks * 16 + kg * 8);
            } else {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    unsigned short t[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) t[q] = as[(ks * 16 + kg * 8 + q) * LDA + wm * TM * 32 + i * 32 + fidx];
                    a[i] = __builtin_bit_cast(bf16x8, t);
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    unsigned short t[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) t[q] = bs[(ks * 16 + kg * 8 + q) * LDB + wn * TN * 32 + j * 32 + fidx];
                    b[j] = __builtin_bit_cast(bf16x8, t);
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if constexpr (EP::kColSum) {          // KRow mode: Bs is [k][n], column sums of dY give the bias gradient
            if (mt == 0 && tid < BN) {
#pragma unroll 8
                for (int k = 0; k < BK; ++k) colsum += bf2f(bs[k * LDB + tid]);
            }
        }
    };
    auto step = [&](int kt, auto stage) {
        constexpr int G = decltype(stage)::value;
        constexpr int GN = (G + 1) % S;
        gload(kt + S, stage);
        compute(kt & 1);
        if (kt + 1 < nk) lstore(std::integral_constant<int, GN>(), (kt + 1) & 1);
        __syncthreads();
    };
    gload(0, std::integral_constant<int, 0>());
    gload(1, std::integral_constant<int, 1>());
    if constexpr (S > 2) gload(2, std::integral_constant<int, 2>());
    if constexpr (S > 3) gload(3, std::integral_constant<int, 3>());
    lstore(std::integral_constant<int, 0>(), 0);
    __syncthreads();
    for (int kt = 0; kt < nk; kt += S) {
        step(kt, std::integral_constant<int, 0>());
        if (kt + 1 < nk) step(kt + 1, std::integral_constant<int, 1>());
        if constexpr (S > 2) { if (kt + 2 < nk) step(kt + 2, std::integral_constant<int, 2>()); }
        if constexpr (S > 3) { if (kt + 3 < nk) step(kt + 3, std::integral_constant<int, 3>()); }
    }

    if constexpr (EP::kColSum) {
        if (mt == 0 && tid < BN && n0 + tid < N) ep.store_colsum(n0 + tid, colsum, z);
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * (TN * 32) + j * 32 + Mma<32>::col(lane);
            typename EP::Aux aux[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * (TM * 32) + i * 32 + Mma<32>::row(r, lane);
                aux[r] = ep.aux(row, col, z, row < M && col < N);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * (TM * 32) + i * 32 + Mma<32>::row(r, lane);
                if (row < M && col < N) ep.store(row, col, acc[i][j][r], z, aux[r]);
            }
        }
}

// ----------------------------------------------------------------------------------------------
// RowK operands (contiguous along k)

// im2col rows of uint8 NCHW states, k = (c, ky, kx): one kernel row of 8 bytes per load; values are
// the bytes themselves (not yet divided by 255).
template <class G> struct ConvU8RowsK8 {
    static_assert(G::KS == 8, "one 8-byte load covers one kernel row");
    static constexpr bool kContig = true;
    typedef uint2 Raw;
    static __device__ __forceinline__ uint4 finish(Raw r, bool ok) { return keep_if_u4(ok, u8x8_to_bf16(r)); }
    const uint8_t* x; int rows;
    struct Fixed { const uint8_t* p; bool ok; };
    __device__ __forceinline__ Fixed prep(int row, int) const {
        Fixed f; f.ok = row < rows;
        row = f.ok ? row : 0;
        const int n = row / (G::HO * G::WO), r = row % (G::HO * G::WO), oy = r / G::WO, ox = r % G::WO;
        f.p = x + (size_t)n * (G::CIN * G::H * G::W) + (oy * G::ST) * G::W + ox * G::ST;
        return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int k, bool pred, bool& ok) const {
        ok = pred && f.ok;
        k = ok ? k : 0;
        const int c = k / 64, ky = (k % 64) / 8;
        const uint32_t* p = reinterpret_cast<const uint32_t*>(f.p + c * (G::H * G::W) + ky * G::W);
        return make_uint2(p[0], p[1]);
    }
};

// im2col rows of a bf16 NHWC activation, k = (ky, kx, c), c in groups of 8.
template <class G> struct ConvNHWCRowsK8 {
    static_assert(G::CIN % 8 == 0, "channels in groups of 8");
    static constexpr bool kContig = true;
    typedef uint4 Raw;
    static __device__ __forceinline__ uint4 finish(Raw r, bool ok) { return keep_if_u4(ok, r); }
    const bf16_t* x; int rows;
    struct Fixed { const bf16_t* p; bool ok; };
    __device__ __forceinline__ Fixed prep(int row, int) const {
        Fixed f; f.ok = row < rows;
        row = f.ok ? row : 0;
        const int n = row / (G::HO * G::WO), r = row % (G::HO * G::WO), oy = r / G::WO, ox = r % G::WO;
        f.p = x + ((size_t)(n * G::H + oy * G::ST) * G::W + ox * G::ST) * G::CIN;
        return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int k, bool pred, bool& ok) const {
        ok = pred && f.ok;
        k = ok ? k : 0;
        const int ky = k / (G::KS * G::CIN), rem = k % (G::KS * G::CIN);
        return *reinterpret_cast<const uint4*>(f.p + ky * (G::W * G::CIN) + rem);
    }
};

struct DenseRowsK8 {            // element (row, k) = base[row*ld + k]
    static constexpr bool kContig = true;
    typedef uint4 Raw;
    static __device__ __forceinline__ uint4 finish(Raw r, bool ok) { return keep_if_u4(ok, r); }
    const bf16_t* base; int rows, ld;
    struct Fixed { const bf16_t* p; bool ok; };
    __device__ __forceinline__ Fixed prep(int row, int) const {
        Fixed f; f.ok = row < rows; f.p = base + (size_t)(f.ok ? row : 0) * ld; return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int k, bool pred, bool& ok) const {
        ok = pred && f.ok;
        return *reinterpret_cast<const uint4*>(f.p + (ok ? k : 0));
    }
};

// Data gradient, gather form (see DgradGatherRowsK): k = (ty, tx, co), co in groups of 8.
template <class G> struct DgradGatherRowsK8 {
    static constexpr bool kContig = true;
    typedef uint4 Raw;
    static __device__ __forceinline__ uint4 finish(Raw r, bool ok) { return keep_if_u4(ok, r); }
    const bf16_t* dy; int rows;
    struct Fixed { const bf16_t* p; int yy, xx; bool ok; };
    __device__ __forceinline__ Fixed prep(int row, int) const {
        Fixed f; f.ok = row < rows;
        row = f.ok ? row : 0;
        const int n = row / (G::HC * G::WC), r = row % (G::HC * G::WC);
        f.yy = r / G::WC; f.xx = r % G::WC;
        f.p = dy + (size_t)n * (G::HO * G::WO * G::COUT);
        return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int k, bool pred, bool& ok) const {
        ok = pred && f.ok;
        k = ok ? k : 0;
        const int tap = k / G::COUT, co = k % G::COUT, ty = tap / G::TAPS, tx = tap % G::TAPS;
        int oy = f.yy - ty, ox = f.xx - tx;
        ok = ok && oy >= 0 && oy < G::HO && ox >= 0 && ox < G::WO;
        oy = ok ? oy : 0; ox = ok ? ox : 0;
        return *reinterpret_cast<const uint4*>(f.p + (oy * G::WO + ox) * G::COUT + co);
    }
};

// Weights seen by the data gradient, from the bf16 copy laid out [ci][ky][kx][co]:
// B(k = (ty,tx,co), n = ci), ky = py + ST*ty, kx = px + ST*tx for parity class z = py*ST + px.
template <class G> struct DgradWeightRowsK8 {
    static constexpr bool kContig = true;
    typedef uint4 Raw;
    static __device__ __forceinline__ uint4 finish(Raw r, bool ok) { return keep_if_u4(ok, r); }
    const bf16_t* w;
    struct Fixed { const bf16_t* p; int py, px; bool ok; };
    __device__ __forceinline__ Fixed prep(int ci, int z) const {
        Fixed f; f.py = z / G::ST; f.px = z % G::ST; f.ok = ci < G::CIN;
        f.p = w + (size_t)(f.ok ? ci : 0) * (G::KS * G::KS * G::COUT);
        return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int k, bool pred, bool& ok) const {
        ok = pred && f.ok;
        k = ok ? k : 0;
        const int tap = k / G::COUT, co = k % G::COUT, ty = tap / G::TAPS, tx = tap % G::TAPS;
        const int ky = f.py + G::ST * ty, kx = f.px + G::ST * tx;
        return *reinterpret_cast<const uint4*>(f.p + (ky * G::KS + kx) * G::COUT + co);
    }
};

// ----------------------------------------------------------------------------------------------
// KRow operands (contiguous along m / n; var = reduction index)

template <class G> struct ConvU8KCols8 {       // A(m = (c,ky,kx), k = output position), 8 kx per load
    static_assert(G::KS == 8, "one 8-byte load covers one kernel row");
    static constexpr bool kContig = false;
    typedef uint2 Raw;
    static __device__ __forceinline__ uint4 finish(Raw r, bool ok) { return keep_if_u4(ok, u8x8_to_bf16(r)); }
    const uint8_t* x; int rows;
    struct Fixed { int off; bool ok; };
    __device__ __forceinline__ Fixed prep(int col, int) const {
        Fixed f; f.ok = col < G::KK;
        col = f.ok ? col : 0;
        const int c = col / 64, ky = (col % 64) / 8;
        f.off = c * (G::H * G::W) + ky * G::W;
        return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int row, bool pred, bool& ok) const {
        ok = pred && f.ok && row < rows;
        row = ok ? row : 0;
        const int n = row / (G::HO * G::WO), r = row % (G::HO * G::WO), oy = r / G::WO, ox = r % G::WO;
        const uint32_t* p = reinterpret_cast<const uint32_t*>(x + (size_t)n * (G::CIN * G::H * G::W) + (oy * G::ST) * G::W + ox * G::ST + f.off);
        return make_uint2(p[0], p[1]);
    }
};

template <class G> struct ConvNHWCKCols8 {     // A(m = (ky,kx,c), k = output position) from bf16 NHWC
    static constexpr bool kContig = false;
    typedef uint4 Raw;
    static __device__ __forceinline__ uint4 finish(Raw r, bool ok) { return keep_if_u4(ok, r); }
    const bf16_t* x; int rows;
    struct Fixed { int off; bool ok; };
    __device__ __forceinline__ Fixed prep(int col, int) const {
        Fixed f; f.ok = col < G::KK;
        col = f.ok ? col : 0;
        const int ky = col / (G::KS * G::CIN), rem = col % (G::KS * G::CIN);
        f.off = ky * (G::W * G::CIN) + rem;
        return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int row, bool pred, bool& ok) const {
        ok = pred && f.ok && row < rows;
        row = ok ? row : 0;
        const int n = row / (G::HO * G::WO), r = row % (G::HO * G::WO), oy = r / G::WO, ox = r % G::WO;
        return *reinterpret_cast<const uint4*>(x + ((size_t)(n * G::H + oy * G::ST) * G::W + ox * G::ST) * G::CIN + f.off);
    }
};

struct DenseKCols8 {            // element (k, col) = base[k*ld + col]
    static constexpr bool kContig = false;
    typedef uint4 Raw;
    static __device__ __forceinline__ uint4 finish(Raw r, bool ok) { return keep_if_u4(ok, r); }
    const bf16_t* base; int cols, ld;
    struct Fixed { const bf16_t* p; bool ok; };
    __device__ __forceinline__ Fixed prep(int col, int) const {
        Fixed f; f.ok = col < cols; f.p = base + (f.ok ? col : 0); return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int k, bool pred, bool& ok) const {
        ok = pred && f.ok;
        return *reinterpret_cast<const uint4*>(f.p + (size_t)(ok ? k : 0) * ld);
    }
};

// ----------------------------------------------------------------------------------------------
// Epilogues with bf16 outputs (EpiPartial of the fp32 core is reused for fp32 partial sums)
struct EpiBiasReluB {           // out[row][col] = bf16(max(scale * v + bias[col], 0))
    static constexpr bool kColSum = false;
    typedef float Aux;
    bf16_t* out; const float* bias; int ldo; float scale;
    __device__ __forceinline__ Aux aux(int, int col, int, bool ok) const { return bias[ok ? col : 0]; }
    __device__ __forceinline__ void store(int row, int col, float v, int, Aux b) const {
        out[(size_t)row * ldo + col] = f2bf(fmaxf(v * scale + b, 0.f));
    }
};

struct EpiPartialScaled {       // out[z][row][col] = scale * v, column sums of B unscaled
    static constexpr bool kColSum = true;
    typedef int Aux;
    float* out; size_t z_stride; int ldo; float* colsum; int colsum_stride; float scale;
    __device__ __forceinline__ Aux aux(int, int, int, bool) const { return 0; }
    __device__ __forceinline__ void store(int row, int col, float v, int z, Aux) const {
        out[z * z_stride + (size_t)row * ldo + col] = v * scale;
    }
    __device__ __forceinline__ void store_colsum(int col, float v, int z) const {
        colsum[(size_t)z * colsum_stride + col] = v;
    }
};

template <class G> struct EpiDgradMaskB {
    static constexpr bool kColSum = false;
    typedef bf16_t Aux;
    bf16_t* dx; const bf16_t* act;
    __device__ __forceinline__ size_t addr(int row, int col, int z) const {
        const int py = z / G::ST, px = z % G::ST;
        const int n = row / (G::HC * G::WC), r = row % (G::HC * G::WC), yy = r / G::WC, xx = r % G::WC;
        return ((size_t)(n * G::H + yy * G::ST + py) * G::W + xx * G::ST + px) * G::CIN + col;
    }
    __device__ __forceinline__ Aux aux(int row, int col, int z, bool ok) const { return act[ok ? addr(row, col, z) : 0]; }
    __device__ __forceinline__ void store(int row, int col, float v, int z, Aux a) const {
        dx[addr(row, col, z)] = (a & 0x7fffu) != 0 && !(a & 0x8000u) ? f2bf(v) : (bf16_t)0;     // act > 0
    }
};

struct EpiDenseMaskB {
    static constexpr bool kColSum = false;
    typedef bf16_t Aux;
    bf16_t* out; const bf16_t* act; int ld;
    __device__ __forceinline__ Aux aux(int row, int col, int, bool ok) const { return act[ok ? (size_t)row * ld + col : 0]; }
    __device__ __forceinline__ void store(int row, int col, float v, int, Aux a) const {
        out[(size_t)row * ld + col] = (a & 0x7fffu) != 0 && !(a & 0x8000u) ? f2bf(v) : (bf16_t)0;
    }
};

template <class T, class AL, class BL, class EP>
inline hipError_t launch_gemm_bf16(hipStream_t s, const AL& al, const BL& bl, const EP& ep, int M, int N, int K,
                                   int z_count, int k_per_split) {
    const int m_tiles = (M + T::BM - 1) / T::BM, n_tiles = (N + T::BN - 1) / T::BN;
    if (M <= 0 || N <= 0 || z_count <= 0) return hipErrorInvalidValue;
    launch_k((gemm_bf16_kernel<T, AL, BL, EP>), dim3(m_tiles * n_tiles, z_count, 1), dim3(256), s, al, bl, ep, M, N, K,
             k_per_split, m_tiles);
    return hipGetLastError();
}

}  // namespace paac
