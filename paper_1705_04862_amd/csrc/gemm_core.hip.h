// Tiled fp32 GEMM core on CDNA4 matrix cores (v_mfma_f32_32x32x2f32 / v_mfma_f32_16x16x4f32)
// with functor-defined operand addressing, used for every dense contraction of the PAAC step:
// convolution forward (implicit im2col rows), data gradient (gather form), weight gradient
// (reduction over output positions, split over workgroups) and the fully connected layer.
//
//   C[m][n] = sum_k A(m,k) * B(k,n)          m < M, n < N, k in this workgroup's k-range
//
// A workgroup of 256 threads (4 wavefronts of 64) owns a BM x BN tile.  Both operands are staged
// through LDS in k-major order (As[k][m], Bs[k][n]) so that the 32 (or 16) lanes that feed one
// MFMA operand read consecutive words: bank-conflict free without swizzling.  An operand whose
// global layout is contiguous along k ("kContig") is transposed on its way into LDS; an operand
// contiguous along m/n is copied with 16-byte stores.  Global loads for k-tile i+1 are issued
// before the MFMAs of k-tile i (register double buffering, two LDS buffers, one barrier per tile).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace paac {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ----------------------------------------------------------------------------------------------
// Wave-level MFMA fragments.  Lane l supplies A[idx = l % MF][k = l / MF] and B[k = l / MF][idx].
template <int MF> struct Mma;
template <> struct Mma<32> {
    typedef f32x16 Acc;
    static constexpr int KSTEP = 2, NACC = 16;
    static __device__ __forceinline__ Acc mma(float a, float b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    // accumulator register r of lane l holds C[row][col]
    static __device__ __forceinline__ int row(int r, int lane) { return (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3); }
    static __device__ __forceinline__ int col(int lane) { return lane & 31; }
};
template <> struct Mma<16> {
    typedef f32x4 Acc;
    static constexpr int KSTEP = 4, NACC = 4;
    static __device__ __forceinline__ Acc mma(float a, float b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int r, int lane) { return (lane >> 4) * 4 + r; }
    static __device__ __forceinline__ int col(int lane) { return lane & 15; }
};

template <int BM_, int BN_, int BK_, int WM_, int WN_, int MF_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MF = MF_;
    static constexpr int TM = BM / (WM * MF), TN = BN / (WN * MF);
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(TM * WM * MF == BM && TN * WN * MF == BN, "tile must be whole fragments");
    static_assert(BK % 4 == 0 && BK % Mma<MF>::KSTEP == 0, "BK granularity");
};

// ----------------------------------------------------------------------------------------------
// Operand functor interface (duck typed):
//   static constexpr bool kContig;
//   struct Fixed;                                   per-thread state of the coordinate that does
//   Fixed prep(int fixed_idx, int z) const;         not change across k-tiles: a row (kContig) or
//                                                   the first of 4 columns (!kContig)
//   float4 load(const Fixed&, int var_idx) const;   kContig: 4 values at k = var_idx .. +3
//                                                   else   : 4 columns at reduction index var_idx
// Out-of-range coordinates return zeros.
// Epilogue: static constexpr bool kColSum; void store(int row, int col, float v, int z) const;
//           void store_colsum(int col, float v, int z) const   (only if kColSum)

template <class T, class AL, class BL, class EP>
__global__ __launch_bounds__(256) void gemm_kernel(const AL al, const BL bl, const EP ep, int M, int N,
                                                   int K, int k_per_split, int m_tiles) {
    typedef Mma<T::MF> MM;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, MF = T::MF, TM = T::TM, TN = T::TN;
    // leading dimensions: odd-ish for transposed scalar stores, multiple of 4 for 16-byte stores
    constexpr int LDA = AL::kContig ? BM + 1 : BM + 4;
    constexpr int LDB = BL::kContig ? BN + 1 : BN + 4;
    constexpr int A_F4 = BM * BK / 4, B_F4 = BN * BK / 4;
    constexpr int A_IT = (A_F4 + 255) / 256, B_IT = (B_F4 + 255) / 256;

    __shared__ __attribute__((aligned(16))) float As[2][BK * LDA];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK * LDB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % T::WM, wn = wave / T::WM;
    const int mt = blockIdx.x % m_tiles, nt = blockIdx.x / m_tiles;
    const int z = blockIdx.y;
    const int m0 = mt * BM, n0 = nt * BN;
    const int k_begin = k_per_split > 0 ? z * k_per_split : 0;
    const int k_end = k_per_split > 0 ? min(K, k_begin + k_per_split) : K;
    const int nk = (k_end - k_begin + BK - 1) / BK;

    // per-thread fixed coordinates of the staging loads
    typename AL::Fixed afix[A_IT];
    typename BL::Fixed bfix[B_IT];
    int a_var[A_IT], a_lds[A_IT], b_var[B_IT], b_lds[B_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        const int f = tid + i * 256;
        if (AL::kContig) {
            const int kq = f % (BK / 4), row = f / (BK / 4);
            afix[i] = al.prep(m0 + row, z);
            a_var[i] = kq * 4;
            a_lds[i] = (kq * 4) * LDA + row;
        } else {
            const int mq = f % (BM / 4), k = f / (BM / 4);
            afix[i] = al.prep(m0 + mq * 4, z);
            a_var[i] = k;
            a_lds[i] = k * LDA + mq * 4;
        }
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
        const int f = tid + i * 256;
        if (BL::kContig) {
            const int kq = f % (BK / 4), col = f / (BK / 4);
            bfix[i] = bl.prep(n0 + col, z);
            b_var[i] = kq * 4;
            b_lds[i] = (kq * 4) * LDB + col;
        } else {
            const int nq = f % (BN / 4), k = f / (BN / 4);
            bfix[i] = bl.prep(n0 + nq * 4, z);
            b_var[i] = k;
            b_lds[i] = k * LDB + nq * 4;
        }
    }

    float4 areg[A_IT], breg[B_IT];
    auto gload = [&](int kt) {
        const int kb = k_begin + kt * BK;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int kk = kb + a_var[i];
            areg[i] = (tid + i * 256 < A_F4 && kk < k_end) ? al.load(afix[i], kk) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const int kk = kb + b_var[i];
            breg[i] = (tid + i * 256 < B_F4 && kk < k_end) ? bl.load(bfix[i], kk) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            if (tid + i * 256 < A_F4) {
                float* p = &As[buf][a_lds[i]];
                if (AL::kContig) { p[0] = areg[i].x; p[LDA] = areg[i].y; p[2 * LDA] = areg[i].z; p[3 * LDA] = areg[i].w; }
                else *reinterpret_cast<float4*>(p) = areg[i];
            }
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            if (tid + i * 256 < B_F4) {
                float* p = &Bs[buf][b_lds[i]];
                if (BL::kContig) { p[0] = breg[i].x; p[LDB] = breg[i].y; p[2 * LDB] = breg[i].z; p[3 * LDB] = breg[i].w; }
                else *reinterpret_cast<float4*>(p) = breg[i];
            }
        }
    };

    typename MM::Acc acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < MM::NACC; ++r) acc[i][j][r] = 0.f;

    float colsum = 0.f;   // used only when EP::kColSum (bias gradient = column sums of B)

    const int fidx = lane % MF, fk = lane / MF;
    const int a_base = wm * (TM * MF) + fidx, b_base = wn * (TN * MF) + fidx;

    if (nk > 0) {
        gload(0);
        lstore(0);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) gload(kt + 1);
        const float* as = As[buf];
        const float* bs = Bs[buf];
#pragma unroll
        for (int ks = 0; ks < BK; ks += MM::KSTEP) {
            float a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = as[(ks + fk) * LDA + a_base + i * MF];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = bs[(ks + fk) * LDB + b_base + j * MF];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = MM::mma(a[i], b[j], acc[i][j]);
        }
        if constexpr (EP::kColSum) {
            if (mt == 0 && tid < BN) {
#pragma unroll 8
                for (int k = 0; k < BK; ++k) colsum += bs[k * LDB + tid];
            }
        }
        if (kt + 1 < nk) lstore(buf ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * (TN * MF) + j * MF + MM::col(lane);
#pragma unroll
            for (int r = 0; r < MM::NACC; ++r) {
                const int row = m0 + wm * (TM * MF) + i * MF + MM::row(r, lane);
                if (row < M && col < N) ep.store(row, col, acc[i][j][r], z);
            }
        }
    if constexpr (EP::kColSum) {
        if (mt == 0 && tid < BN && n0 + tid < N) ep.store_colsum(n0 + tid, colsum, z);
    }
}

// ----------------------------------------------------------------------------------------------
// Geometry of one convolution layer (valid padding), all compile-time.
template <int CIN_, int H_, int W_, int KS_, int ST_, int COUT_>
struct ConvGeom {
    static constexpr int CIN = CIN_, H = H_, W = W_, KS = KS_, ST = ST_, COUT = COUT_;
    static constexpr int HO = (H - KS) / ST + 1, WO = (W - KS) / ST + 1;
    static constexpr int KK = KS * KS * CIN;             // im2col row length
    // data gradient in gather form: input positions are split into ST*ST parity classes, each
    // sees TAPS x TAPS kernel taps
    static constexpr int TAPS = KS / ST, HC = (H + ST - 1) / ST, WC = (W + ST - 1) / ST;
    static constexpr int KD = TAPS * TAPS * COUT;
    static_assert(KS % ST == 0, "kernel must be a multiple of the stride");
    static_assert(H % ST == 0 && W % ST == 0, "parity classes must be equal-sized");
};

__device__ __forceinline__ float4 zero4() { return make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ float4 u8x4_to_unit(uint32_t w) {
    const float s = 1.0f / 255.0f;
    return make_float4((float)(w & 255u) * s, (float)((w >> 8) & 255u) * s, (float)((w >> 16) & 255u) * s,
                       (float)(w >> 24) * s);
}

// im2col rows of a uint8 NCHW image batch, k = (c, ky, kx); value = byte / 255.
template <class G> struct ConvU8RowsK {
    static constexpr bool kContig = true;
    const uint8_t* x; int rows;
    struct Fixed { const uint8_t* p; };
    __device__ __forceinline__ Fixed prep(int row, int) const {
        Fixed f; f.p = nullptr;
        if (row < rows) {
            const int n = row / (G::HO * G::WO), r = row % (G::HO * G::WO), oy = r / G::WO, ox = r % G::WO;
            f.p = x + (size_t)n * (G::CIN * G::H * G::W) + (oy * G::ST) * G::W + ox * G::ST;
        }
        return f;
    }
    __device__ __forceinline__ float4 load(const Fixed& f, int k) const {
        if (!f.p) return zero4();
        const int c = k / (G::KS * G::KS), r = k % (G::KS * G::KS), ky = r / G::KS, kx = r % G::KS;
        return u8x4_to_unit(*reinterpret_cast<const uint32_t*>(f.p + c * (G::H * G::W) + ky * G::W + kx));
    }
};

// im2col rows of a float NHWC activation, k = (ky, kx, c).
template <class G> struct ConvNHWCRowsK {
    static constexpr bool kContig = true;
    const float* x; int rows;
    struct Fixed { const float* p; };
    __device__ __forceinline__ Fixed prep(int row, int) const {
        Fixed f; f.p = nullptr;
        if (row < rows) {
            const int n = row / (G::HO * G::WO), r = row % (G::HO * G::WO), oy = r / G::WO, ox = r % G::WO;
            f.p = x + ((size_t)(n * G::H + oy * G::ST) * G::W + ox * G::ST) * G::CIN;
        }
        return f;
    }
    __device__ __forceinline__ float4 load(const Fixed& f, int k) const {
        if (!f.p) return zero4();
        const int ky = k / (G::KS * G::CIN), rem = k % (G::KS * G::CIN);
        return *reinterpret_cast<const float4*>(f.p + ky * (G::W * G::CIN) + rem);
    }
};

// Row-major matrix read along its rows: element (row, k) = base[row*ld + k].
struct DenseRowsK {
    static constexpr bool kContig = true;
    const float* base; int rows, ld;
    struct Fixed { const float* p; };
    __device__ __forceinline__ Fixed prep(int row, int) const {
        Fixed f; f.p = row < rows ? base + (size_t)row * ld : nullptr; return f;
    }
    __device__ __forceinline__ float4 load(const Fixed& f, int k) const {
        return f.p ? *reinterpret_cast<const float4*>(f.p + k) : zero4();
    }
};

// Row-major matrix read along its columns: element (k, col) = base[k*ld + col].
struct DenseKCols {
    static constexpr bool kContig = false;
    const float* base; int cols, ld;
    struct Fixed { const float* p; };
    __device__ __forceinline__ Fixed prep(int col, int) const {
        Fixed f; f.p = col < cols ? base + col : nullptr; return f;
    }
    __device__ __forceinline__ float4 load(const Fixed& f, int k) const {
        return f.p ? *reinterpret_cast<const float4*>(f.p + (size_t)k * ld) : zero4();
    }
};

// Data gradient, gather form.  Row = (n, yy, xx) of parity class z = (py, px); k = (ty, tx, co);
// value = dY[n][yy - ty][xx - tx][co] when that output position exists, else 0.
template <class G> struct DgradGatherRowsK {
    static constexpr bool kContig = true;
    const float* dy; int rows;
    struct Fixed { const float* p; int yy, xx; };
    __device__ __forceinline__ Fixed prep(int row, int) const {
        Fixed f; f.p = nullptr; f.yy = 0; f.xx = 0;
        if (row < rows) {
            const int n = row / (G::HC * G::WC), r = row % (G::HC * G::WC);
            f.yy = r / G::WC; f.xx = r % G::WC;
            f.p = dy + (size_t)n * (G::HO * G::WO * G::COUT);
        }
        return f;
    }
    __device__ __forceinline__ float4 load(const Fixed& f, int k) const {
        if (!f.p) return zero4();
        const int tap = k / G::COUT, co = k % G::COUT, ty = tap / G::TAPS, tx = tap % G::TAPS;
        const int oy = f.yy - ty, ox = f.xx - tx;
        if (oy < 0 || oy >= G::HO || ox < 0 || ox >= G::WO) return zero4();
        return *reinterpret_cast<const float4*>(f.p + (oy * G::WO + ox) * G::COUT + co);
    }
};

// Weights seen by the data gradient: B(k = (ty,tx,co), n = ci) = W[(ky,kx,ci)][co] with
// ky = py + ST*ty, kx = px + ST*tx for parity class z = py*ST + px.
template <class G> struct DgradWeightColsK {
    static constexpr bool kContig = true;
    const float* w;
    struct Fixed { const float* p; int py, px; };
    __device__ __forceinline__ Fixed prep(int ci, int z) const {
        Fixed f; f.py = z / G::ST; f.px = z % G::ST;
        f.p = ci < G::CIN ? w + (size_t)ci * G::COUT : nullptr;
        return f;
    }
    __device__ __forceinline__ float4 load(const Fixed& f, int k) const {
        if (!f.p) return zero4();
        const int tap = k / G::COUT, co = k % G::COUT, ty = tap / G::TAPS, tx = tap % G::TAPS;
        const int ky = f.py + G::ST * ty, kx = f.px + G::ST * tx;
        return *reinterpret_cast<const float4*>(f.p + (size_t)(ky * G::KS + kx) * (G::CIN * G::COUT) + co);
    }
};

// Weight gradient of the first layer: A(m = (c,ky,kx), k = output position) = byte / 255.
template <class G> struct ConvU8KCols {
    static constexpr bool kContig = false;
    const uint8_t* x; int rows;
    struct Fixed { int off; };
    __device__ __forceinline__ Fixed prep(int col, int) const {
        Fixed f; f.off = -1;
        if (col < G::KK) {
            const int c = col / (G::KS * G::KS), r = col % (G::KS * G::KS), ky = r / G::KS, kx = r % G::KS;
            f.off = c * (G::H * G::W) + ky * G::W + kx;
        }
        return f;
    }
    __device__ __forceinline__ float4 load(const Fixed& f, int row) const {
        if (f.off < 0 || row >= rows) return zero4();
        const int n = row / (G::HO * G::WO), r = row % (G::HO * G::WO), oy = r / G::WO, ox = r % G::WO;
        const uint8_t* p = x + (size_t)n * (G::CIN * G::H * G::W) + (oy * G::ST) * G::W + ox * G::ST + f.off;
        return u8x4_to_unit(*reinterpret_cast<const uint32_t*>(p));
    }
};

// Weight gradient of the later conv layers: A(m = (ky,kx,c), k = output position) from NHWC input.
template <class G> struct ConvNHWCKCols {
    static constexpr bool kContig = false;
    const float* x; int rows;
    struct Fixed { int off; };
    __device__ __forceinline__ Fixed prep(int col, int) const {
        Fixed f; f.off = -1;
        if (col < G::KK) {
            const int ky = col / (G::KS * G::CIN), rem = col % (G::KS * G::CIN);
            f.off = ky * (G::W * G::CIN) + rem;
        }
        return f;
    }
    __device__ __forceinline__ float4 load(const Fixed& f, int row) const {
        if (f.off < 0 || row >= rows) return zero4();
        const int n = row / (G::HO * G::WO), r = row % (G::HO * G::WO), oy = r / G::WO, ox = r % G::WO;
        return *reinterpret_cast<const float4*>(x + ((size_t)(n * G::H + oy * G::ST) * G::W + ox * G::ST) * G::CIN + f.off);
    }
};

// ----------------------------------------------------------------------------------------------
// Epilogues
struct EpiBiasRelu {            // out[row][col] = max(v + bias[col], 0)
    static constexpr bool kColSum = false;
    float* out; const float* bias; int ldo;
    __device__ __forceinline__ void store(int row, int col, float v, int) const {
        out[(size_t)row * ldo + col] = fmaxf(v + bias[col], 0.f);
    }
};

template <bool COLSUM> struct EpiPartial {   // out[z][row][col] = v ; optional column sums of B
    static constexpr bool kColSum = COLSUM;
    float* out; size_t z_stride; int ldo; float* colsum; int colsum_stride;
    __device__ __forceinline__ void store(int row, int col, float v, int z) const {
        out[z * z_stride + (size_t)row * ldo + col] = v;
    }
    __device__ __forceinline__ void store_colsum(int col, float v, int z) const {
        colsum[(size_t)z * colsum_stride + col] = v;
    }
};

template <class G> struct EpiDgradMask {     // scatter a parity class back to NHWC, times ReLU'
    static constexpr bool kColSum = false;
    float* dx; const float* act;
    __device__ __forceinline__ void store(int row, int col, float v, int z) const {
        const int py = z / G::ST, px = z % G::ST;
        const int n = row / (G::HC * G::WC), r = row % (G::HC * G::WC), yy = r / G::WC, xx = r % G::WC;
        const size_t a = ((size_t)(n * G::H + yy * G::ST + py) * G::W + xx * G::ST + px) * G::CIN + col;
        dx[a] = act[a] > 0.f ? v : 0.f;
    }
};

struct EpiDenseMask {           // out[row][col] = act[row][col] > 0 ? v : 0
    static constexpr bool kColSum = false;
    float* out; const float* act; int ld;
    __device__ __forceinline__ void store(int row, int col, float v, int) const {
        const size_t a = (size_t)row * ld + col;
        out[a] = act[a] > 0.f ? v : 0.f;
    }
};

// ----------------------------------------------------------------------------------------------
template <class T, class AL, class BL, class EP>
inline hipError_t launch_gemm(hipStream_t s, const AL& al, const BL& bl, const EP& ep, int M, int N, int K,
                              int z_count, int k_per_split) {
    const int m_tiles = (M + T::BM - 1) / T::BM, n_tiles = (N + T::BN - 1) / T::BN;
    if (M <= 0 || N <= 0 || z_count <= 0) return hipErrorInvalidValue;
    dim3 grid(m_tiles * n_tiles, z_count, 1);
    hipLaunchKernelGGL((gemm_kernel<T, AL, BL, EP>), grid, dim3(256), 0, s, al, bl, ep, M, N, K, k_per_split, m_tiles);
    return hipGetLastError();
}

}  // namespace paac
