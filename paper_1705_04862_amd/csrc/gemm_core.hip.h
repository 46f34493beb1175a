// Tiled fp32 GEMM core on CDNA4 matrix cores (v_mfma_f32_32x32x2f32)
// with functor-defined operand addressing, used for every dense contraction of the PAAC step:
// convolution forward (implicit im2col rows), data gradient (gather form), weight gradient
// (reduction over output positions, split over workgroups) and the fully connected layer.
//
//   C[m][n] = sum_k A(m,k) * B(k,n)          m < M, n < N, k in this workgroup's k-range
//
// A workgroup of 4 (or 8) wavefronts of 64 owns a BM x BN tile.  Both operands are staged
// through LDS.  An operand whose global layout is contiguous along k ("kContig") is kept row-major,
// [row][BK + 4]: one 16-byte store per thread and one 16-byte fragment read per lane and four MFMA
// steps (a lane takes four consecutive k; the order in which the k of a tile are multiplied is free).
// An operand contiguous along m/n is kept k-major, [k][rows + 4], copied with 16-byte stores and read
// word by word (32 consecutive lanes read consecutive words).  Global loads run S k-tiles ahead of the
// MFMAs through S register stages (two LDS buffers, one barrier per tile): these layers are bound by
// memory latency, not bandwidth, at the paper's batch sizes.  MFMA fragments are 32x32x2 or, for the
// smallest launches, 16x16x4.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "internal.h"
#include <type_traits>
#include <utility>

namespace paac {

typedef float f32x16 __attribute__((ext_vector_type(16)));

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
typedef float f32x4 __attribute__((ext_vector_type(4)));
template <> struct Mma<16> {              // 16 x 16 x 4, 32 cycles: the same rate in a quarter of the output
    typedef f32x4 Acc;
    static constexpr int KSTEP = 4, NACC = 4;
    static __device__ __forceinline__ Acc mma(float a, float b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int r, int lane) { return (lane >> 4) * 4 + r; }
    static __device__ __forceinline__ int col(int lane) { return lane & 15; }
};
// BM x BN x BK tile; the four waves are arranged WM (along m) x WN (along n) x WK (along k): with
// WK > 1 several waves accumulate the same output fragments over different k-steps of every tile
// and their accumulators are added through LDS before the epilogue.  This keeps four MFMA pipes
// busy on a tile as small as 32 x 32, which the small-batch layers need.
template <int BM_, int BN_, int BK_, int WM_, int WN_, int WK_, int MF_, int STAGES_ = 3>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, WK = WK_, MF = MF_, STAGES = STAGES_;
    static constexpr int NT = WM * WN * WK * 64;             // threads of the workgroup
    static_assert(STAGES >= 2 && STAGES <= 4, "register prefetch depth");
    static constexpr int TM = BM / (WM * MF), TN = BN / (WN * MF);
    static_assert(WM * WN * WK == 4 || WM * WN * WK == 8, "four or eight wavefronts per workgroup");
    static_assert((BK / Mma<MF>::KSTEP) % WK == 0, "k-steps must divide among the k-waves");
    static_assert(TM * WM * MF == BM && TN * WN * MF == BN, "tile must be whole fragments");
    static_assert(BK % 4 == 0 && BK % Mma<MF>::KSTEP == 0, "BK granularity");
};

// ----------------------------------------------------------------------------------------------
// Operand functor interface (duck typed):
//   static constexpr bool kContig;
//   struct Fixed;                                   per-thread state of the coordinate that does
//   Fixed prep(int fixed_idx, int z) const;         not change across k-tiles: a row (kContig) or
//                                                   the first of 4 columns (!kContig)
//   Raw load(const Fixed&, int var_idx, bool pred, bool& ok) const;
//                                                   kContig: 4 values at k = var_idx .. +3
//                                                   else   : 4 columns at reduction index var_idx
//     always issues the load from a clamped, valid address (branch free) and reports in `ok`
//     whether the coordinate was in range (and pred held);
//   static float4 finish(Raw, bool ok);             conversion + zeroing, applied when the registers
//                                                   are written to LDS
// Epilogue: static constexpr bool kColSum; typedef Aux;
//           Aux aux(int row, int col, int z, bool ok) const;      auxiliary load (bias / mask), clamped
//           void store(int row, int col, float v, int z, Aux) const;
//           void store_colsum(int col, float v, int z) const      (only if kColSum)

template <class E, class = void> struct AuxEarly { static constexpr bool value = false; };
template <class E> struct AuxEarly<E, std::enable_if_t<E::kAuxEarly>> { static constexpr bool value = true; };
// Epilogues whose element address is a sum of a row part and a column part declare kSplitAddr and give
//   int row_part(int row, int z) const; int col_part(int col, int z) const;   (element offsets)
//   const float* mask() const; float* dst() const;      out[rp + cp] = mask[rp + cp] > 0 ? v : 0
// A thread then computes 16 row parts and one column part per fragment instead of the address of every
// element twice (its divisions by the geometry's constants were most of a scatter epilogue's instructions).
template <class E, class = void> struct SplitAddr { static constexpr bool value = false; };
template <class E> struct SplitAddr<E, std::enable_if_t<E::kSplitAddr>> { static constexpr bool value = true; };
template <class L, class = void> struct RowFast { static constexpr bool value = false; };
template <class L> struct RowFast<L, std::enable_if_t<L::kRowFast>> { static constexpr bool value = true; };
template <class L> __host__ __device__ constexpr bool row_fast() { return RowFast<L>::value; }

// LDS floats of one workgroup: two buffers per operand.  An operand that is contiguous along k in
// memory (kContig) is kept row-major, [row][BK + 4]: a thread stores its four k with one 16-byte store
// and a lane reads four k of its fragment row with one 16-byte read (the pad makes the pitch an odd
// multiple of 16 bytes: sixteen rows fall into sixteen different bank groups).  The others are
// contiguous along the row and are kept k-major, [k][rows + 4].
template <class T, class AL, class BL> constexpr int gemm_smem_floats() {
    return 2 * (AL::kContig ? T::BM * (T::BK + 4) : T::BK * (T::BM + 4)) +
           2 * (BL::kContig ? T::BN * (T::BK + 4) : T::BK * (T::BN + 4));
}

// One workgroup's share of a GEMM: output tile `tile_idx` (m tiles fastest), k-split `z`.
template <class T, class AL, class BL, class EP>
__device__ __forceinline__ void gemm_body(const AL& al, const BL& bl, const EP& ep, int M, int N, int K, int k_per_split,
                                          int m_tiles, int tile_idx, int z, float* smem) {
    typedef Mma<T::MF> MM;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, MF = T::MF, TM = T::TM, TN = T::TN;
    // leading dimensions (floats): row pitch of a row-major operand, k pitch of a k-major one
    constexpr int LDA = AL::kContig ? BK + 4 : BM + 4;
    constexpr int LDB = BL::kContig ? BK + 4 : BN + 4;
    constexpr int A_F4 = BM * BK / 4, B_F4 = BN * BK / 4;
    constexpr int NT = T::NT;
    constexpr int A_IT = (A_F4 + NT - 1) / NT, B_IT = (B_F4 + NT - 1) / NT;

    constexpr int A_BUF = AL::kContig ? BM * LDA : BK * LDA;      // floats per LDS buffer (multiples of 4)
    constexpr int B_BUF = BL::kContig ? BN * LDB : BK * LDB;
    static_assert(2 * A_BUF + 2 * B_BUF == gemm_smem_floats<T, AL, BL>(), "LDS size");
    float* const As = smem;                 // As[buf] = As + buf * A_BUF
    float* const Bs = smem + 2 * A_BUF;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % T::WM, wn = (wave / T::WM) % T::WN, wk = wave / (T::WM * T::WN);
    const int mt = tile_idx % m_tiles, nt = tile_idx / m_tiles;
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
        const int f = tid + i * NT;
        if (AL::kContig) {
            // consecutive lanes take consecutive k of a row, or (kRowFast) consecutive rows at one k:
            // whichever walks contiguous memory for this operand
            const int kq = row_fast<AL>() ? f / BM : f % (BK / 4), row = row_fast<AL>() ? f % BM : f / (BK / 4);
            afix[i] = al.prep(m0 + row, z);
            a_var[i] = kq * 4;
            a_lds[i] = row * LDA + kq * 4;
        } else {
            const int mq = f % (BM / 4), k = f / (BM / 4);
            afix[i] = al.prep(m0 + mq * 4, z);
            a_var[i] = k;
            a_lds[i] = k * LDA + mq * 4;
        }
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
        const int f = tid + i * NT;
        if (BL::kContig) {
            const int kq = f % (BK / 4), col = f / (BK / 4);
            bfix[i] = bl.prep(n0 + col, z);
            b_var[i] = kq * 4;
            b_lds[i] = col * LDB + kq * 4;
        } else {
            const int nq = f % (BN / 4), k = f / (BN / 4);
            bfix[i] = bl.prep(n0 + nq * 4, z);
            b_var[i] = k;
            b_lds[i] = k * LDB + nq * 4;
        }
    }

    // S register stages: k-tile j travels through stage j % S; while tile i is multiplied the global
    // loads of tiles i+1 .. i+S are in flight
    // The loaded registers are not touched (no conversion, no zeroing) until they are stored to LDS:
    // any earlier use would make the wavefront wait for the load it has just issued.
    constexpr int S = T::STAGES;
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
            areg[G][i] = al.load(afix[i], kk, (A_F4 % NT == 0 || tid + i * NT < A_F4) && kk < k_end, ok);
            bits |= ok ? (1u << i) : 0u;
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const int kk = kb + b_var[i];
            bool ok;
            breg[G][i] = bl.load(bfix[i], kk, (B_F4 % NT == 0 || tid + i * NT < B_F4) && kk < k_end, ok);
            bits |= ok ? (1u << (16 + i)) : 0u;
        }
        okbits[G] = bits;
    };
    // register stage -> LDS buffer, one staging unit (u < A_IT: operand A, else operand B)
    auto lstore_unit = [&](auto stage, int buf, auto unit) {
        constexpr int G = decltype(stage)::value;
        constexpr int u = decltype(unit)::value;
        if constexpr (u < A_IT) {
            constexpr int i = u;
            if (A_F4 % NT == 0 || tid + i * NT < A_F4) {
                float* p = As + buf * A_BUF + a_lds[i];
                const float4 v = AL::finish(areg[G][i], (okbits[G] >> i) & 1u);
                *reinterpret_cast<float4*>(p) = v;
            }
        } else {
            constexpr int i = u - A_IT;
            if (B_F4 % NT == 0 || tid + i * NT < B_F4) {
                float* p = Bs + buf * B_BUF + b_lds[i];
                const float4 v = BL::finish(breg[G][i], (okbits[G] >> (16 + i)) & 1u);
                *reinterpret_cast<float4*>(p) = v;
            }
        }
    };
    auto lstore = [&](auto stage, int buf) {
        [&]<int... U>(std::integer_sequence<int, U...>) {
            (lstore_unit(stage, buf, std::integral_constant<int, U>()), ...);
        }(std::make_integer_sequence<int, A_IT + B_IT>());
    };

    // a wave with a single output fragment alternates between two accumulators so that consecutive
    // MFMAs do not wait on each other; the two are added in the epilogue
    constexpr int KACC = (TM * TN == 1) ? 2 : 1;
    typename MM::Acc acc[KACC][TM][TN];
#pragma unroll
    for (int q = 0; q < KACC; ++q)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < MM::NACC; ++r) acc[q][i][j][r] = 0.f;

    float colsum = 0.f;   // used only when EP::kColSum (bias gradient = column sums of B)

    const int fidx = lane % MF, fk = lane / MF;
    const int a_base = wm * (TM * MF) + fidx, b_base = wn * (TN * MF) + fidx;

    // The MFMAs of the current tile with the LDS stores of the next tile in between.  An fp32 MFMA
    // holds the matrix pipe for 64 cycles and a wave issues in order: the conversion and store work
    // of one staging unit placed after an MFMA runs in its shadow instead of after the last MFMA
    // (at small batch a wave has its SIMD to itself, nothing else would fill the gap).  The
    // scheduling barriers keep the compiler from regrouping it.
    constexpr int NS = BK / MM::KSTEP / T::WK;      // k-steps of this wave
    static_assert(NS % 4 == 0, "k-steps are taken in groups of four");
    constexpr int UNITS = A_IT + B_IT;
    static_assert(UNITS <= NS, "at most one staging unit per k-step");
    auto compute_and_store = [&](int buf, auto stage_next, int buf_next) {
        const float* as = As + buf * A_BUF;
        const float* bs = Bs + buf * B_BUF;
        // every LDS read of the tile is issued before the first MFMA: one LDS latency per tile
        // instead of one per group of MFMAs
        // k-wave wk owns the k range [wk NS KSTEP, (wk + 1) NS KSTEP) of the tile; within it MFMA step
        // 4 g + j of lane-group fk multiplies k = 4 KSTEP g + 4 fk + j (any order of k is a valid dot
        // product as long as both operands use it): four consecutive k per lane and group of four steps
        float a[NS][TM], b[NS][TN];
#pragma unroll
        for (int g = 0; g < NS / 4; ++g) {
            const int k0 = (wk * NS + 4 * g) * MM::KSTEP + 4 * fk;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if constexpr (AL::kContig) {
                    const float4 v = *reinterpret_cast<const float4*>(as + (a_base + i * MF) * LDA + k0);
                    a[4 * g][i] = v.x; a[4 * g + 1][i] = v.y; a[4 * g + 2][i] = v.z; a[4 * g + 3][i] = v.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) a[4 * g + j][i] = as[(k0 + j) * LDA + a_base + i * MF];
                }
            }
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                if constexpr (BL::kContig) {
                    const float4 v = *reinterpret_cast<const float4*>(bs + (b_base + i * MF) * LDB + k0);
                    b[4 * g][i] = v.x; b[4 * g + 1][i] = v.y; b[4 * g + 2][i] = v.z; b[4 * g + 3][i] = v.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) b[4 * g + j][i] = bs[(k0 + j) * LDB + b_base + i * MF];
                }
            }
        }
        [&]<int... ST>(std::integer_sequence<int, ST...>) {
            ([&] {
                constexpr int st = ST;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int q = st % KACC;
                        acc[q][i][j] = MM::mma(a[st][i], b[st][j], acc[q][i][j]);
                    }
                // staging unit u goes after k-step u * NS / UNITS (spread evenly, the first right away)
                constexpr int u = (st * UNITS + NS - 1) / NS;
                if constexpr (u < UNITS && (u * NS) / UNITS == st) {
                    __builtin_amdgcn_sched_barrier(0);
                    lstore_unit(stage_next, buf_next, std::integral_constant<int, u>());
                    __builtin_amdgcn_sched_barrier(0);
                }
            }(), ...);
        }(std::make_integer_sequence<int, NS>());
        if constexpr (EP::kColSum) {
            if (mt == 0 && tid < BN) {
#pragma unroll 8
                for (int k = 0; k < BK; ++k) colsum += BL::kContig ? bs[tid * LDB + k] : bs[k * LDB + tid];
            }
        }
    };

    // one pipeline step for the tile in register-stage position G (= kt % S)
    auto step = [&](int kt, auto stage) {
        constexpr int G = decltype(stage)::value;
        constexpr int GN = (G + 1) % S;
        gload(kt + S, stage);      // stage G was stored to LDS one step ago; past the end: clamped, zeroed
        compute_and_store(kt & 1, std::integral_constant<int, GN>(), (kt + 1) & 1);   // after the last tile: zeros nobody reads
        __syncthreads();
    };
    // Auxiliary epilogue operands (bias, ReLU mask) do not depend on the accumulators: their loads are
    // issued before the first operand load, so the epilogue does not start with a memory round trip
    // (about a microsecond, a tenth of a small-batch kernel).
    typename EP::Aux aux[TM][TN][MM::NACC];
    auto load_aux = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn * (TN * MF) + j * MF + MM::col(lane);
#pragma unroll
                for (int r = 0; r < MM::NACC; ++r) {
                    const int row = m0 + wm * (TM * MF) + i * MF + MM::row(r, lane);
                    aux[i][j][r] = ep.aux(row, col, z, wk == 0 && row < M && col < N);
                }
            }
    };
    if constexpr (AuxEarly<EP>::value) load_aux();      // one register per column (a bias); masks would cost 16
    // Scatter epilogues with a mask (data gradients): the addresses and the mask values of the wave's fragments
    // are fetched before the first operand load where a wave owns one fragment (16 registers each), so that the
    // epilogue, which is on the critical path of the fused backward launches, does not start with a memory round
    // trip; with more fragments per wave they are fetched after the k loop.
    int sat[SplitAddr<EP>::value ? TM : 1][TN][MM::NACC];
    float smk[SplitAddr<EP>::value ? TM : 1][TN][MM::NACC];
    constexpr bool MASK_EARLY = TM * TN == 1;         // two fragments per wave (64 registers): measured slower, 31.7 -> 38.1 us
    auto load_masks = [&]() __attribute__((always_inline)) {
      if constexpr (SplitAddr<EP>::value) {
        int cp[TN]; bool cok[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * (TN * MF) + j * MF + MM::col(lane);
            cok[j] = col < N;
            cp[j] = ep.col_part(cok[j] ? col : 0, z);
        }
        const float* const mk = ep.mask();
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < MM::NACC; ++r) {
                const int row = m0 + wm * (TM * MF) + i * MF + MM::row(r, lane);
                const bool rok = wk == 0 && row < M;
                const int rp = ep.row_part(rok ? row : 0, z);
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    sat[i][j][r] = rok && cok[j] ? rp + cp[j] : -1;
                    smk[i][j][r] = mk[sat[i][j][r] >= 0 ? sat[i][j][r] : 0];
                }
            }
      }
    };
    if constexpr (SplitAddr<EP>::value && MASK_EARLY) load_masks();
    gload(0, std::integral_constant<int, 0>());
    gload(1, std::integral_constant<int, 1>());
    if constexpr (S > 2) gload(2, std::integral_constant<int, 2>());
    if constexpr (S > 3) gload(3, std::integral_constant<int, 3>());
    lstore(std::integral_constant<int, 0>(), 0);
    __syncthreads();
    // Whole rounds of S steps run without any branch, the remainder after the loop.  With a step that
    // can be skipped inside the loop the compiler sees a path on which a register stage is loaded
    // again while its previous load is still outstanding, and waits for ALL loads at the loop head:
    // that would drain the prefetch pipeline once per round.
    int kt = 0;
    for (int q = nk / S; q > 0; --q, kt += S) {
        step(kt, std::integral_constant<int, 0>());
        step(kt + 1, std::integral_constant<int, 1>());
        if constexpr (S > 2) step(kt + 2, std::integral_constant<int, 2>());
        if constexpr (S > 3) step(kt + 3, std::integral_constant<int, 3>());
    }
    if (kt < nk) {
        step(kt, std::integral_constant<int, 0>());
        if (kt + 1 < nk) {
            step(kt + 1, std::integral_constant<int, 1>());
            if constexpr (S > 2) { if (kt + 2 < nk) step(kt + 2, std::integral_constant<int, 2>()); }
        }
    }

    if constexpr (EP::kColSum) {
        if (mt == 0 && tid < BN && n0 + tid < N) ep.store_colsum(n0 + tid, colsum, z);
    }
    if constexpr (KACC == 2) {
#pragma unroll
        for (int r = 0; r < MM::NACC; ++r) acc[0][0][0][r] += acc[1][0][0][r];
    }
    if constexpr (T::WK > 1) {
        // add the accumulators of the k-waves: waves wk > 0 park theirs in LDS (the staging buffers are
        // free now: the loop ended with a barrier), wave wk == 0 of each (wm, wn) adds them and stores
        constexpr int PER_WAVE = TM * TN * MM::NACC * 64;
        static_assert((T::WK - 1) * T::WM * T::WN * PER_WAVE <= 2 * A_BUF + 2 * B_BUF, "reduction scratch must fit the staging buffers");
        float* red = smem;
        if (wk > 0) {
            float* dst = red + ((wk - 1) * (T::WM * T::WN) + (wave % (T::WM * T::WN))) * PER_WAVE + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < MM::NACC; ++r) dst[((i * TN + j) * MM::NACC + r) * 64] = acc[0][i][j][r];
        }
        __syncthreads();
        if (wk > 0) return;
#pragma unroll
        for (int q = 1; q < T::WK; ++q) {
            const float* src = red + ((q - 1) * (T::WM * T::WN) + wave) * PER_WAVE + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < MM::NACC; ++r) acc[0][i][j][r] += src[((i * TN + j) * MM::NACC + r) * 64];
        }
    }
    if constexpr (SplitAddr<EP>::value) {
        if constexpr (!MASK_EARLY) load_masks();
        float* const out = ep.dst();
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < MM::NACC; ++r)
                    if (sat[i][j][r] >= 0) out[sat[i][j][r]] = smk[i][j][r] > 0.f ? acc[0][i][j][r] : 0.f;
        return;
    }
    if constexpr (!AuxEarly<EP>::value) load_aux();     // every auxiliary load of the tile, then the stores
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * (TN * MF) + j * MF + MM::col(lane);
#pragma unroll
            for (int r = 0; r < MM::NACC; ++r) {
                const int row = m0 + wm * (TM * MF) + i * MF + MM::row(r, lane);
                if (row < M && col < N) ep.store(row, col, acc[0][i][j][r], z, aux[i][j][r]);
            }
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
__device__ __forceinline__ float4 keep_if(bool ok, float4 v) {
    return make_float4(ok ? v.x : 0.f, ok ? v.y : 0.f, ok ? v.z : 0.f, ok ? v.w : 0.f);
}
// All loaders are branch free: an out-of-range coordinate is clamped to a valid address, the load
// is always issued, and the value is replaced by zero afterwards.  (A load under a branch makes the
// compiler wait for every outstanding load at the join, which would serialise the prefetch stages.)
//   load(fixed, var, ok): `ok` = the caller's own predicate (k-range, tile bounds)

// im2col rows of a float NHWC activation, k = (ky, kx, c).
template <class G> struct ConvNHWCRowsK {
    static constexpr bool kContig = true;
    typedef float4 Raw;
    static __device__ __forceinline__ float4 finish(Raw r, bool ok) { return keep_if(ok, r); }
    const float* x; int rows;
    struct Fixed { const float* p; bool ok; };
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
        return *reinterpret_cast<const float4*>(f.p + ky * (G::W * G::CIN) + rem);
    }
};

// Row-major matrix read along its rows: element (row, k) = base[row*ld + k].
struct DenseRowsK {
    static constexpr bool kContig = true;
    typedef float4 Raw;
    static __device__ __forceinline__ float4 finish(Raw r, bool ok) { return keep_if(ok, r); }
    const float* base; int rows, ld;
    struct Fixed { const float* p; bool ok; };
    __device__ __forceinline__ Fixed prep(int row, int) const {
        Fixed f; f.ok = row < rows; f.p = base + (size_t)(f.ok ? row : 0) * ld; return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int k, bool pred, bool& ok) const {
        ok = pred && f.ok;
        return *reinterpret_cast<const float4*>(f.p + (ok ? k : 0));
    }
};

// Row-major matrix read along its columns: element (k, col) = base[k*ld + col].
struct DenseKCols {
    static constexpr bool kContig = false;
    typedef float4 Raw;
    static __device__ __forceinline__ float4 finish(Raw r, bool ok) { return keep_if(ok, r); }
    const float* base; int cols, ld;
    struct Fixed { const float* p; bool ok; };
    __device__ __forceinline__ Fixed prep(int col, int) const {
        Fixed f; f.ok = col < cols; f.p = base + (f.ok ? col : 0); return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int k, bool pred, bool& ok) const {
        ok = pred && f.ok;
        return *reinterpret_cast<const float4*>(f.p + (size_t)(ok ? k : 0) * ld);
    }
};

// Data gradient, gather form.  Row = (n, yy, xx) of parity class z = (py, px); k = (ty, tx, co);
// value = dY[n][yy - ty][xx - tx][co] when that output position exists, else 0.
template <class G> struct DgradGatherRowsK {
    static constexpr bool kContig = true;
    typedef float4 Raw;
    static __device__ __forceinline__ float4 finish(Raw r, bool ok) { return keep_if(ok, r); }
    const float* dy; int rows;
    struct Fixed { const float* p; int yy, xx; bool ok; };
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
        return *reinterpret_cast<const float4*>(f.p + (oy * G::WO + ox) * G::COUT + co);
    }
};

// Weights seen by the data gradient: B(k = (ty,tx,co), n = ci) = W[(ky,kx,ci)][co] with
// ky = py + ST*ty, kx = px + ST*tx for parity class z = py*ST + px.
template <class G> struct DgradWeightColsK {
    static constexpr bool kContig = true;
    typedef float4 Raw;
    static __device__ __forceinline__ float4 finish(Raw r, bool ok) { return keep_if(ok, r); }
    const float* w;
    struct Fixed { const float* p; int py, px; bool ok; };
    __device__ __forceinline__ Fixed prep(int ci, int z) const {
        Fixed f; f.py = z / G::ST; f.px = z % G::ST; f.ok = ci < G::CIN;
        f.p = w + (size_t)(f.ok ? ci : 0) * G::COUT;
        return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int k, bool pred, bool& ok) const {
        ok = pred && f.ok;
        k = ok ? k : 0;
        const int tap = k / G::COUT, co = k % G::COUT, ty = tap / G::TAPS, tx = tap % G::TAPS;
        const int ky = f.py + G::ST * ty, kx = f.px + G::ST * tx;
        return *reinterpret_cast<const float4*>(f.p + (size_t)(ky * G::KS + kx) * (G::CIN * G::COUT) + co);
    }
};

// The same with all ST*ST parity classes as columns, n = (z, ci): the classes of one block of input
// positions read the same gathered dY rows, so one GEMM with N = ST*ST*CIN gathers them once.
template <class G> struct DgradWeightColsKAll {
    static constexpr bool kContig = true;
    typedef float4 Raw;
    static __device__ __forceinline__ float4 finish(Raw r, bool ok) { return keep_if(ok, r); }
    const float* w;
    struct Fixed { const float* p; int py, px; bool ok; };
    __device__ __forceinline__ Fixed prep(int col, int) const {
        Fixed f; f.ok = col < G::ST * G::ST * G::CIN;
        col = f.ok ? col : 0;
        const int z = col / G::CIN, ci = col % G::CIN;
        f.py = z / G::ST; f.px = z % G::ST;
        f.p = w + (size_t)ci * G::COUT;
        return f;
    }
    __device__ __forceinline__ Raw load(const Fixed& f, int k, bool pred, bool& ok) const {
        ok = pred && f.ok;
        k = ok ? k : 0;
        const int tap = k / G::COUT, co = k % G::COUT, ty = tap / G::TAPS, tx = tap % G::TAPS;
        const int ky = f.py + G::ST * ty, kx = f.px + G::ST * tx;
        return *reinterpret_cast<const float4*>(f.p + (size_t)(ky * G::KS + kx) * (G::CIN * G::COUT) + co);
    }
};

// Weight gradient of the later conv layers: A(m = (ky,kx,c), k = output position) from NHWC input.
template <class G> struct ConvNHWCKCols {
    static constexpr bool kContig = false;
    typedef float4 Raw;
    static __device__ __forceinline__ float4 finish(Raw r, bool ok) { return keep_if(ok, r); }
    const float* x; int rows;
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
        return *reinterpret_cast<const float4*>(x + ((size_t)(n * G::H + oy * G::ST) * G::W + ox * G::ST) * G::CIN + f.off);
    }
};

// ----------------------------------------------------------------------------------------------
// Epilogues
struct EpiBiasRelu {            // out[row][col] = max(v + bias[col], 0)
    static constexpr bool kColSum = false, kAuxEarly = true;
    typedef float Aux;
    float* out; const float* bias; int ldo;
    __device__ __forceinline__ Aux aux(int, int col, int, bool) const { return bias[col < ldo ? col : 0]; }   // one load per column
    __device__ __forceinline__ void store(int row, int col, float v, int, Aux b) const {
        out[(size_t)row * ldo + col] = fmaxf(v + b, 0.f);
    }
};

template <bool COLSUM> struct EpiPartial {   // out[z][row][col] = v ; optional column sums of B
    static constexpr bool kColSum = COLSUM;
    typedef int Aux;
    float* out; size_t z_stride; int ldo; float* colsum; int colsum_stride;
    __device__ __forceinline__ Aux aux(int, int, int, bool) const { return 0; }
    __device__ __forceinline__ void store(int row, int col, float v, int z, Aux) const {
        out[z * z_stride + (size_t)row * ldo + col] = v;
    }
    __device__ __forceinline__ void store_colsum(int col, float v, int z) const {
        colsum[(size_t)z * colsum_stride + col] = v;
    }
};

template <class G> struct EpiDgradMask {     // scatter a parity class back to NHWC, times ReLU'
    static constexpr bool kColSum = false, kSplitAddr = true;
    typedef float Aux;
    float* dx; const float* act;
    __device__ __forceinline__ int row_part(int row, int) const {
        const int n = row / (G::HC * G::WC), r = row % (G::HC * G::WC), yy = r / G::WC, xx = r % G::WC;
        return ((n * G::H + yy * G::ST) * G::W + xx * G::ST) * G::CIN;
    }
    __device__ __forceinline__ int col_part(int col, int z) const { return ((z / G::ST) * G::W + z % G::ST) * G::CIN + col; }
    __device__ __forceinline__ const float* mask() const { return act; }
    __device__ __forceinline__ float* dst() const { return dx; }
    __device__ __forceinline__ size_t addr(int row, int col, int z) const {
        const int py = z / G::ST, px = z % G::ST;
        const int n = row / (G::HC * G::WC), r = row % (G::HC * G::WC), yy = r / G::WC, xx = r % G::WC;
        return ((size_t)(n * G::H + yy * G::ST + py) * G::W + xx * G::ST + px) * G::CIN + col;
    }
    __device__ __forceinline__ Aux aux(int row, int col, int z, bool ok) const { return act[ok ? addr(row, col, z) : 0]; }
    __device__ __forceinline__ void store(int row, int col, float v, int z, Aux a) const {
        dx[addr(row, col, z)] = a > 0.f ? v : 0.f;
    }
};

template <class G> struct EpiDgradMaskAll {  // the same for columns n = (z, ci) of all parity classes
    static constexpr bool kColSum = false, kSplitAddr = true;
    typedef float Aux;
    float* dx; const float* act;
    __device__ __forceinline__ int row_part(int row, int) const {
        const int n = row / (G::HC * G::WC), r = row % (G::HC * G::WC), yy = r / G::WC, xx = r % G::WC;
        return ((n * G::H + yy * G::ST) * G::W + xx * G::ST) * G::CIN;
    }
    __device__ __forceinline__ int col_part(int col, int) const {
        const int z = col / G::CIN, ci = col % G::CIN;
        return ((z / G::ST) * G::W + z % G::ST) * G::CIN + ci;
    }
    __device__ __forceinline__ const float* mask() const { return act; }
    __device__ __forceinline__ float* dst() const { return dx; }
    __device__ __forceinline__ size_t addr(int row, int col) const {
        const int z = col / G::CIN, ci = col % G::CIN, py = z / G::ST, px = z % G::ST;
        const int n = row / (G::HC * G::WC), r = row % (G::HC * G::WC), yy = r / G::WC, xx = r % G::WC;
        return ((size_t)(n * G::H + yy * G::ST + py) * G::W + xx * G::ST + px) * G::CIN + ci;
    }
    __device__ __forceinline__ Aux aux(int row, int col, int, bool ok) const { return act[ok ? addr(row, col) : 0]; }
    __device__ __forceinline__ void store(int row, int col, float v, int, Aux a) const {
        dx[addr(row, col)] = a > 0.f ? v : 0.f;
    }
};

struct EpiDenseMask {           // out[row][col] = act[row][col] > 0 ? v : 0
    static constexpr bool kColSum = false, kSplitAddr = true;
    typedef float Aux;
    float* out; const float* act; int ld;
    __device__ __forceinline__ int row_part(int row, int) const { return row * ld; }
    __device__ __forceinline__ int col_part(int col, int) const { return col; }
    __device__ __forceinline__ const float* mask() const { return act; }
    __device__ __forceinline__ float* dst() const { return out; }
    __device__ __forceinline__ Aux aux(int row, int col, int, bool ok) const { return act[ok ? (size_t)row * ld + col : 0]; }
    __device__ __forceinline__ void store(int row, int col, float v, int, Aux a) const {
        out[(size_t)row * ld + col] = a > 0.f ? v : 0.f;
    }
};

// ----------------------------------------------------------------------------------------------
// Workgroup ids are dealt round-robin to the eight XCDs, each with an L2 of its own.  xcd_order
// renumbers them so that the workgroups of one XCD take consecutive positions in the tile order:
// neighbours there share an operand slice, and now they share an L2 as well (measured: HBM-side
// traffic falls, time by 1-6 % on the fc GEMMs and not at all on the small convolutions).
__device__ __forceinline__ int xcd_order(int id, int total) {
    const int x = id & 7, q = total >> 3, r = total & 7;
    return x * q + min(x, r) + (id >> 3);
}

template <class T, class AL, class BL, class EP>
__global__ __launch_bounds__(T::NT) void gemm_kernel(const AL al, const BL bl, const EP ep, int M, int N,
                                                   int K, int k_per_split, int m_tiles) {
    __shared__ __attribute__((aligned(16))) float smem[gemm_smem_floats<T, AL, BL>()];
    int id = blockIdx.x + gridDim.x * blockIdx.y;         // dispatch order: x fastest
    id = xcd_order(id, gridDim.x * gridDim.y);
    gemm_body<T, AL, BL, EP>(al, bl, ep, M, N, K, k_per_split, m_tiles, id % (int)gridDim.x, id / (int)gridDim.x, smem);
}

// A GEMM with its launch shape, as a value: lets two independent GEMMs share one launch.
template <class T_, class AL_, class BL_, class EP_> struct GemmCall {
    typedef T_ T; typedef AL_ AL; typedef BL_ BL; typedef EP_ EP;
    AL al; BL bl; EP ep;
    int M, N, K, z_count, k_per_split;
    __host__ __device__ int m_tiles() const { return (M + T::BM - 1) / T::BM; }
    __host__ __device__ int tiles() const { return m_tiles() * ((N + T::BN - 1) / T::BN); }
    __host__ __device__ int blocks() const { return tiles() * z_count; }
};
template <class T, class AL, class BL, class EP>
inline GemmCall<T, AL, BL, EP> make_call(const AL& al, const BL& bl, const EP& ep, int M, int N, int K, int z, int k_per) {
    return GemmCall<T, AL, BL, EP>{al, bl, ep, M, N, K, z, k_per};
}

// Two independent GEMMs in one grid: workgroups [0, a.blocks()) run `a`, the rest run `b`.  At small
// batch each GEMM alone leaves most compute units idle and is bound by its own start-up and drain
// latencies; side by side they overlap them.
template <class C1, class C2>
__global__ __launch_bounds__(256) void gemm_pair_kernel(const C1 a, const C2 b) {
    static_assert(C1::T::NT == 256 && C2::T::NT == 256, "both halves run on four wavefronts");
    constexpr int S1 = gemm_smem_floats<typename C1::T, typename C1::AL, typename C1::BL>();
    constexpr int S2 = gemm_smem_floats<typename C2::T, typename C2::AL, typename C2::BL>();
    __shared__ __attribute__((aligned(16))) float smem[S1 > S2 ? S1 : S2];
    const int n1 = a.blocks();
    if ((int)blockIdx.x < n1) {
        const int t = a.tiles();
        const int id = xcd_order(blockIdx.x, n1);
        gemm_body<typename C1::T, typename C1::AL, typename C1::BL, typename C1::EP>(
            a.al, a.bl, a.ep, a.M, a.N, a.K, a.k_per_split, a.m_tiles(), id % t, id / t, smem);
    } else {
        const int t = b.tiles();
        const int r = xcd_order(blockIdx.x - n1, (int)gridDim.x - n1);
        gemm_body<typename C2::T, typename C2::AL, typename C2::BL, typename C2::EP>(
            b.al, b.bl, b.ep, b.M, b.N, b.K, b.k_per_split, b.m_tiles(), r % t, r / t, smem);
    }
}

template <class C1, class C2>
inline hipError_t launch_pair(hipStream_t s, const C1& a, const C2& b) {
    if (a.blocks() <= 0 || b.blocks() <= 0) return hipErrorInvalidValue;
    launch_k((gemm_pair_kernel<C1, C2>), dim3(a.blocks() + b.blocks(), 1, 1), dim3(256), s, a, b);
    return hipGetLastError();
}

template <class T, class AL, class BL, class EP>
inline hipError_t launch_gemm(hipStream_t s, const AL& al, const BL& bl, const EP& ep, int M, int N, int K,
                              int z_count, int k_per_split) {
    const int m_tiles = (M + T::BM - 1) / T::BM, n_tiles = (N + T::BN - 1) / T::BN;
    if (M <= 0 || N <= 0 || z_count <= 0) return hipErrorInvalidValue;
    dim3 grid(m_tiles * n_tiles, z_count, 1);
    launch_k((gemm_kernel<T, AL, BL, EP>), grid, dim3(T::NT), s, al, bl, ep, M, N, K, k_per_split, m_tiles);
    return hipGetLastError();
}

}  // namespace paac
