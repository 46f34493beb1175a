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
//        contiguous along m / n in memory; a thread loads 8 columns at 4 consecutive reduction
//        indices, transposes the 8 x 4 block in registers (byte permutes) and stores it into the
//        same [row][BK] LDS layout, so the MFMA side is identical in both modes.
// Global loads are 16 bytes (8 bf16; 8 bytes for the uint8 first layer), branch free and clamped,
// S register stages ahead; conversion and zeroing happen when the registers are stored to LDS.
#pragma once
#include "gemm_core.hip.h"
#include <algorithm>

namespace paac {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ bf16_t f2bf(float f) { __bf16 b = (__bf16)f; return __builtin_bit_cast(unsigned short, b); }
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float((unsigned)h << 16); }
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2v __attribute__((ext_vector_type(2)));
// both conversions as one vector conversion: a single v_cvt_pk_bf16_f32 (the two scalar conversions
// became two of them plus a shift and an OR); same rounding
__device__ __forceinline__ unsigned pack2(float lo, float hi) {
    const f32x2v v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
// acc + lo + hi of a packed bf16 pair: one v_dot2 against (1, 1)
__device__ __forceinline__ float dot2_ones(unsigned pair, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc, false);
}
__device__ __forceinline__ bool bf16_positive(bf16_t a) { return (a & 0x7fffu) != 0 && !(a & 0x8000u); }
// keep the bf16 halves of v whose counterpart in a is a positive number: as a signed 16-bit integer a
// positive bf16 (NaN with a clear sign bit included, as above) is > 0; three packed 16-bit operations
// (clamp below at 0, above at 1, times 0xffff) and the AND instead of two compare chains per half
typedef short i16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned mask2(unsigned v, unsigned a) {
    const i16x2 zero = {0, 0}, one = {1, 1};
    const i16x2 pos = __builtin_elementwise_min(__builtin_elementwise_max(__builtin_bit_cast(i16x2, a), zero), one);    // 1 where a > 0
    const u16x2 all = {0xffffu, 0xffffu};
    return v & __builtin_bit_cast(unsigned, (u16x2)(__builtin_bit_cast(u16x2, pos) * all));
}

// staging registers as a native vector type: an array of the uint4 struct that is only copied in and
// out is lowered to memcpy through private memory (scratch) instead of registers
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 zero_u4() { return make_uint4(0u, 0u, 0u, 0u); }
// The value lane ^ 1 holds: a DPP move inside the quad.  (__shfl_xor goes through the LDS crossbar and is
// waited for like an LDS read: 24 such round trips were 3 000 of the 8 700 cycles a sample took in the
// third layer's data gradient.)  Every lane of the wave must be active.
__device__ __forceinline__ float lane_xor1(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
}
// Row pitch of an LDS image whose rows an MFMA A fragment walks: lane m reads 16 bytes of the m-th
// position, positions are `pos_chunks` 16-byte chunks apart (odd: sixteen consecutive positions of a
// row hit the sixteen 16-byte bank groups once), and after `lanes_per_row` positions the fragment
// continues in the next image row.  A ds_read_b128 is served sixteen consecutive lanes per cycle; with
// the natural row pitch the lanes behind a row end land on bank groups that lanes before it use
// (measured: 8-10 cycles per fragment read instead of 4.4).  Returned: the smallest pitch (elements,
// a multiple of eight) >= min_elems that continues the bank sequence across the row end, i.e. whose
// chunk count is lanes_per_row * pos_chunks modulo 16.
constexpr int bank_continuing_pitch(int min_elems, int lanes_per_row, int pos_chunks) {
    int c = (min_elems + 7) / 8;
    while (c % 16 != (lanes_per_row * pos_chunks) % 16) ++c;
    return c * 8;
}
// Waves that split the k-steps of one 32-wide column block add their 32 x 32 accumulators through LDS.
// Every wave of the KW finishes its own groups of four accumulator registers (group g of a fragment =
// rows 8 g + 4 (lane / 32) .. + 3): it hands the other waves' groups over as 16-byte stores, and after
// the workgroup's barrier adds what the others left for it, in wave order whichever wave adds.  With
// the first wave of a block adding and finishing everything, the others idled through the longest
// part of a sample (2 000 of 7 500 cycles in the third layer's data gradient).
template <int NB, int KW, int FRAGS> struct KShares {
    static_assert(KW == 1 || KW == 2 || KW == 4, "groups of four registers divide evenly");
    static constexpr int GPO = 4 / KW;                 // groups per owner and fragment
    static constexpr int FLOATS = NB * KW * (KW - 1) * FRAGS * GPO * 64 * 4;
    static __device__ __forceinline__ int slot(int nb, int owner, int src, int f, int gi, int lane) {
        return (((((nb * KW + owner) * (KW - 1) + (src - (src > owner ? 1 : 0))) * FRAGS + f) * GPO + gi) * 64 + lane) * 4;
    }
    template <int KG> static __device__ __forceinline__ void give(const f32x16 (&acc)[FRAGS], float* red, int nb, int lane) {
#pragma unroll
        for (int o = 0; o < KW; ++o)
            if (o != KG) {
#pragma unroll
                for (int f = 0; f < FRAGS; ++f)
#pragma unroll
                    for (int gi = 0; gi < GPO; ++gi) {
                        const int g = o * GPO + gi;
                        const f32x4 v = {acc[f][4 * g], acc[f][4 * g + 1], acc[f][4 * g + 2], acc[f][4 * g + 3]};
                        *reinterpret_cast<f32x4*>(red + slot(nb, o, KG, f, gi, lane)) = v;
                    }
            }
    }
    // after the barrier: the sums of wave KG's groups, in acc[f][4 g ..] for g = KG * GPO + gi
    template <int KG> static __device__ __forceinline__ void take(f32x16 (&acc)[FRAGS], const float* red, int nb, int lane) {
        if constexpr (KW > 1) {
            f32x4 got[KW - 1][FRAGS][GPO];
#pragma unroll
            for (int src = 0; src < KW; ++src)
                if (src != KG) {
#pragma unroll
                    for (int f = 0; f < FRAGS; ++f)
#pragma unroll
                        for (int gi = 0; gi < GPO; ++gi)
                            got[src - (src > KG ? 1 : 0)][f][gi] = *reinterpret_cast<const f32x4*>(red + slot(nb, KG, src, f, gi, lane));
                }
#pragma unroll
            for (int f = 0; f < FRAGS; ++f)
#pragma unroll
                for (int gi = 0; gi < GPO; ++gi) {
                    const int g = KG * GPO + gi;
                    const f32x4 own = {acc[f][4 * g], acc[f][4 * g + 1], acc[f][4 * g + 2], acc[f][4 * g + 3]};
                    f32x4 t = KG == 0 ? own : got[0][f][gi];
#pragma unroll
                    for (int src = 1; src < KW; ++src) t += src == KG ? own : got[src - (src > KG ? 1 : 0)][f][gi];
                    acc[f][4 * g] = t.x; acc[f][4 * g + 1] = t.y; acc[f][4 * g + 2] = t.z; acc[f][4 * g + 3] = t.w;
                }
        }
    }
};
// runs fn(std::integral_constant<int, kg>) for the wave-uniform kg in [0, KW): accumulator indices stay constants
template <int KW, class F> __device__ __forceinline__ void with_k_share(int kg, F&& fn) {
    if (kg == 0) fn(std::integral_constant<int, 0>());
    if constexpr (KW > 1) { if (kg == 1) fn(std::integral_constant<int, 1>()); }
    if constexpr (KW > 2) {
        if (kg == 2) fn(std::integral_constant<int, 2>());
        if (kg == 3) fn(std::integral_constant<int, 3>());
    }
}
__device__ __forceinline__ uint4 keep_if_u4(bool ok, uint4 v) {
    return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
}
// eight bytes -> eight bf16 holding the byte values 0..255 exactly (8 significand bits suffice);
// the 1/255 of the input scaling is applied to the fp32 accumulators in the epilogue instead, so the
// first layer's input carries no rounding error at all.  An integer below 256 has zero low fp32
// mantissa bits: its bf16 is the upper half of the fp32, so two conversions pack with one byte permute.
__device__ __forceinline__ unsigned u8pair_to_bf16(float lo, float hi) {
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}
__device__ __forceinline__ uint4 u8x8_to_bf16(uint2 w) {
    auto cv = [&](unsigned x, int sh) { return (float)((x >> sh) & 255u); };
    return make_uint4(u8pair_to_bf16(cv(w.x, 0), cv(w.x, 8)), u8pair_to_bf16(cv(w.x, 16), cv(w.x, 24)),
                      u8pair_to_bf16(cv(w.y, 0), cv(w.y, 8)), u8pair_to_bf16(cv(w.y, 16), cv(w.y, 24)));
}

template <int BM_, int BN_, int BK_, int WM_, int WN_, int STAGES_ = 3, int MINW_ = 2>
struct TileB {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, STAGES = STAGES_;
    static constexpr int MINW = MINW_;                       // waves per SIMD the register budget is sized for
    static constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(TM * WM * 32 == BM && TN * WN * 32 == BN, "tile must be whole 32x32 fragments");
    static_assert(BK % 16 == 0, "BK must be a multiple of the MFMA depth");
};

// Operand functor interface (8-wide):
//   static constexpr bool kContig;      true: RowK operand (fixed = row, var = k, multiple of 8)
//                                       false: KRow operand (fixed = first of 8 columns, var = k)
//   typedef Raw; Raw load(fixed, var, pred, ok&);  static uint4 finish(Raw, ok)  -> 8 bf16
//
// LDS layout, both modes: tile[row][BK + 8].  The 16 bytes of padding per row make 16 consecutive
// rows start in 16 different groups of four banks (row pitch 36 words, 64 banks): the 16-byte reads
// of the MFMA side (lanes along rows) are conflict free, as measured with SQ_LDS_BANK_CONFLICT; an
// XOR permutation of the chunks on top of the padding was measured to cause conflicts (45-55% of the
// LDS cycles) and is not used.  The transposing store of the KRow mode (8-byte stores, lanes along
// k) touches 2 words x 16 lanes x 2 row groups = all 64 banks once.
//
// Persistent workgroups: the grid's x extent may be smaller than the number of output tiles; a
// workgroup walks tiles blockIdx.x, blockIdx.x + gridDim.x, ... (the hardware starts only ~90
// workgroups per microsecond, so one workgroup per 128-row tile of a large batch would be bound by
// that rate).  The load pipeline is refilled per tile on purpose: global stores inside the k loop
// would share the wave's memory counter with the prefetched loads, and every wait would then have
// to drain the whole pipeline; the refill latency is covered by the other workgroups of the CU.
// Epilogue flavours: the fp32 core's epilogues take (row, col) and store from the accumulator layout;
// epilogues declared with kEntry produce a bf16 tile that is addressed by a per-row entry (an element
// offset from row_entry(row, z), optionally through the LDS row table) plus a column offset.
template <class EP, class = void> struct EpiTraits { static constexpr bool kEntry = false, kRowTable = false; };
template <class EP> struct EpiTraits<EP, std::enable_if_t<EP::kEntry>> {
    static constexpr bool kEntry = true, kRowTable = EP::kRowTable;
};
// KRow loaders whose address needs divisions per reduction index (im2col of an output position)
// declare kRowTab: the kernel then keeps the per-index offsets of the coming k tiles in a small LDS
// table, filled by 64 threads one pipeline step ahead, and a staging unit fetches its four offsets
// with one 16-byte LDS read instead of four chains of integer divisions.
template <class L, class = void> struct RowTab { static constexpr bool value = false; };
template <class L> struct RowTab<L, std::enable_if_t<L::kRowTab>> { static constexpr bool value = true; };

template <class EP, class = void> struct EpiColMap {          // column index -> offset added to the row entry
    static __device__ __forceinline__ int off(const EP&, int col) { return col; }
};
template <class EP> struct EpiColMap<EP, std::enable_if_t<EP::kColMap>> {
    static __device__ __forceinline__ int off(const EP& ep, int col) { return ep.col_off(col); }
};

template <class T, class AL, class BL, class EP>
__global__ __launch_bounds__(256, T::MINW) void gemm_bf16_kernel(const AL al, const BL bl, const EP ep, int M, int N, int K,
                                                        int k_per_split, int m_tiles, int n_tiles, int group_m,
                                                        int z_count) {
    static_assert(AL::kContig == BL::kContig, "both operands use the same staging mode");
    constexpr bool ROWK = AL::kContig;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, TM = T::TM, TN = T::TN, S = T::STAGES;
    constexpr int LD = BK + 8;                                   // bf16 elements per LDS row
    constexpr int A_BUF = BM * LD, B_BUF = BN * LD;
    constexpr int NL = ROWK ? 1 : 4;                             // global loads per staging unit
    // staging unit: RowK = one 16-byte chunk of one row; KRow = 8 rows x 4 reduction indices
    constexpr int A_U = ROWK ? BM * BK / 8 : (BM / 8) * (BK / 4);
    constexpr int B_U = ROWK ? BN * BK / 8 : (BN / 8) * (BK / 4);
    constexpr int A_IT = (A_U + 255) / 256, B_IT = (B_U + 255) / 256;
    static_assert((A_IT + B_IT) * NL <= 32, "ok-bit mask");
    // Side jobs of the weight-gradient mode are spread over the waves so that no wave is the
    // straggler of every step: the B staging units (fewer than 256) go to the last waves, the
    // row-offset table is filled by wave 0, the bias-gradient column sums by wave 1.
    constexpr int B_SHIFT = (!ROWK && B_U % 256 != 0) ? 256 - B_U % 256 : 0;
    constexpr int CS0 = ROWK ? 0 : 64;

    __shared__ __attribute__((aligned(16))) bf16_t smem[2 * A_BUF + 2 * B_BUF];
    // epilogues whose output address needs divisions per row (scatter of a parity class) get the BM
    // row entries of a tile computed once, by BM threads, into a table (two copies: a wave may start
    // the next tile while another still stores the previous one)
    __shared__ int rowtab[EpiTraits<EP>::kRowTable ? 2 * BM : 1];
    bf16_t* const As = smem;
    bf16_t* const Bs = smem + 2 * A_BUF;
    constexpr bool ATAB = !ROWK && RowTab<AL>::value;
    constexpr int RS = S + 1;                                     // table slots: k tile j lives in slot j % RS
    __shared__ __attribute__((aligned(16))) int ktab[ATAB ? RS * BK : 4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % T::WM, wn = wave / T::WM;
    const int tiles = m_tiles * n_tiles;
    // Which tile(s) and k-split this workgroup owns.  Default: tiles blockIdx.x, + gridDim.x, ...;
    // split blockIdx.y.  With group_m > 0 the grid is one-dimensional, one tile per workgroup, and
    // workgroups that read the same operand slices (group_m consecutive m tiles x all n tiles of
    // one k-split) are placed on the same XCD, next to each other in its dispatch order: workgroup
    // ids go round-robin over the 8 XCDs, each with its own L2, so without this the shared slices
    // are fetched from HBM once per XCD (measured 1-2% L2 hit rate in the weight-gradient GEMMs).
    int z = blockIdx.y, c_tile = blockIdx.x, tile_stride = gridDim.x;
    if (group_m > 0) {
        const int gsz = group_m * n_tiles, mblocks = m_tiles / group_m;
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int idx = slot % gsz, g = (slot / gsz) * 8 + xcd;
        if (g >= mblocks * z_count) return;                      // padding of the last round of 8 groups
        z = g / mblocks;
        c_tile = (g % mblocks) * group_m + idx % group_m + m_tiles * (idx / group_m);
        tile_stride = tiles;                                     // exactly one tile
    }
    const int k_begin = k_per_split > 0 ? z * k_per_split : 0;
    const int k_end = k_per_split > 0 ? min(K, k_begin + k_per_split) : K;
    const int nk = (k_end - k_begin + BK - 1) / BK;
    if (nk <= 0 || c_tile >= tiles) return;

    // ---- staging units of this thread: tile-independent part
    int a_var[A_IT], a_lds[A_IT], a_fix0[A_IT], b_var[B_IT], b_lds[B_IT], b_fix0[B_IT];
    auto unit = [&](int f, int rows, bool rowfast, int& fix0, int& var, int& lds) __attribute__((always_inline)) {
        if (ROWK) {
            int c = rowfast ? f / rows : f % (BK / 8);
            const int row = rowfast ? f % rows : f / (BK / 8);
            // lanes along the rows: the 64 lanes of a wave share the chunk, so everything that depends
            // on k (kernel tap, channel offset, range test) is computed once per wave on the scalar unit
            if (rowfast && rows % 64 == 0) c = __builtin_amdgcn_readfirstlane(c);
            fix0 = row; var = c * 8; lds = row * LD + c * 8;
        } else {
            const int kq = f % (BK / 4), cq = f / (BK / 4);          // lanes along k: conflict-free 8-byte LDS stores
            fix0 = cq * 8; var = kq * 4; lds = cq * 8 * LD + kq * 4;
        }
    };
#pragma unroll
    for (int i = 0; i < A_IT; ++i) unit(tid + i * 256, BM, row_fast<AL>(), a_fix0[i], a_var[i], a_lds[i]);
#pragma unroll
    for (int i = 0; i < B_IT; ++i) unit(max(tid + i * 256 - B_SHIFT, 0), BN, row_fast<BL>(), b_fix0[i], b_var[i], b_lds[i]);   // non-owners: a valid unit, predicated off
    // does this thread own B staging unit i?
    auto b_on = [&](int i) __attribute__((always_inline)) {
        return B_U % 256 == 0 || (tid + i * 256 >= B_SHIFT && tid + i * 256 - B_SHIFT < B_U);
    };

    typename AL::Fixed afix[A_IT];
    typename BL::Fixed bfix[B_IT];
    auto set_load_tile = [&](int tile) __attribute__((always_inline)) {
        const int m0 = (tile % m_tiles) * BM, n0 = (tile / m_tiles) * BN;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) afix[i] = al.prep(m0 + a_fix0[i], z);
#pragma unroll
        for (int i = 0; i < B_IT; ++i) bfix[i] = bl.prep(n0 + b_fix0[i], z);
    };

    // offsets of the reduction indices of k tile `kt` (also past the end: -1 = load nothing)
    auto fill_tab = [&](int kt, int idx) __attribute__((always_inline)) {
        if constexpr (ATAB) {
            const int r = k_begin + kt * BK + idx;
            ktab[(kt % RS) * BK + idx] = r < k_end ? al.row_entry(r) : -1;
        }
    };
    typename AL::Raw areg[S][A_IT][NL];
    typename BL::Raw breg[S][B_IT][NL];
    unsigned okbits[S];
    auto gload = [&](int kt, auto stage) __attribute__((always_inline)) {     // kt past the end: predicated off
        constexpr int G = decltype(stage)::value;
        const int kb = k_begin + kt * BK;
        unsigned bits = 0;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            if constexpr (ATAB) {
                const int4 e = *reinterpret_cast<const int4*>(&ktab[(kt % RS) * BK + a_var[i]]);
                const int ent[4] = {e.x, e.y, e.z, e.w};
#pragma unroll
                for (int q = 0; q < NL; ++q) {
                    bool ok;
                    areg[G][i][q] = al.load_at(afix[i], ent[q], A_U % 256 == 0 || tid + i * 256 < A_U, ok);
                    bits |= ok ? (1u << (i * NL + q)) : 0u;
                }
            } else {
#pragma unroll
                for (int q = 0; q < NL; ++q) {
                    const int kk = kb + a_var[i] + q;
                    bool ok;
                    areg[G][i][q] = al.load(afix[i], kk, (A_U % 256 == 0 || tid + i * 256 < A_U) && kk < k_end, ok);
                    bits |= ok ? (1u << (i * NL + q)) : 0u;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i)
#pragma unroll
            for (int q = 0; q < NL; ++q) {
                const int kk = kb + b_var[i] + q;
                bool ok;
                breg[G][i][q] = bl.load(bfix[i], kk, b_on(i) && kk < k_end, ok);
                bits |= ok ? (1u << ((A_IT + i) * NL + q)) : 0u;
            }
        okbits[G] = bits;
    };
    // registers of one unit -> LDS.  KRow: r[q] holds columns c..c+7 at reduction index k+q; column j
    // gets the four values {r[0][j], r[1][j], r[2][j], r[3][j]} as one 8-byte store.
    auto put = [&](bf16_t* dst, const uint4 (&r)[NL]) {
        if constexpr (ROWK) {
            *reinterpret_cast<uint4*>(dst) = r[0];
        } else {
            const unsigned w[4][4] = {{r[0].x, r[0].y, r[0].z, r[0].w}, {r[1].x, r[1].y, r[1].z, r[1].w},
                                      {r[2].x, r[2].y, r[2].z, r[2].w}, {r[3].x, r[3].y, r[3].z, r[3].w}};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const unsigned sel = (j & 1) ? 0x07060302u : 0x05040100u;
                uint2 o;
                o.x = __builtin_amdgcn_perm(w[1][j >> 1], w[0][j >> 1], sel);
                o.y = __builtin_amdgcn_perm(w[3][j >> 1], w[2][j >> 1], sel);
                *reinterpret_cast<uint2*>(dst + j * LD) = o;
            }
        }
    };
    // register stage -> LDS buffer, one staging unit (u < A_IT: operand A, else operand B)
    auto lstore_unit = [&](auto stage, int buf, auto unit) __attribute__((always_inline)) {
        constexpr int G = decltype(stage)::value;
        constexpr int u = decltype(unit)::value;
        if constexpr (u < A_IT) {
            constexpr int i = u;
            if (A_U % 256 == 0 || tid + i * 256 < A_U) {
                uint4 r[NL];
#pragma unroll
                for (int q = 0; q < NL; ++q) r[q] = AL::finish(areg[G][i][q], (okbits[G] >> (i * NL + q)) & 1u);
                put(As + buf * A_BUF + a_lds[i], r);
            }
        } else {
            constexpr int i = u - A_IT;
            if (b_on(i)) {
                uint4 r[NL];
#pragma unroll
                for (int q = 0; q < NL; ++q) r[q] = BL::finish(breg[G][i][q], (okbits[G] >> ((A_IT + i) * NL + q)) & 1u);
                put(Bs + buf * B_BUF + b_lds[i], r);
            }
        }
    };
    auto lstore = [&](auto stage, int buf) __attribute__((always_inline)) {
        [&]<int... U>(std::integer_sequence<int, U...>) {
            (lstore_unit(stage, buf, std::integral_constant<int, U>()), ...);
        }(std::make_integer_sequence<int, A_IT + B_IT>());
    };

    f32x16 acc[TM][TN];
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    };
    zero_acc();
    float colsum = 0.f;

    const int fidx = lane & 31, kg = lane >> 5;
    int tile_par = 0;
    // MFMAs of the current k tile with the LDS stores of the next one spread between the four
    // 16-deep sub-steps (the stores' conversion / permute work runs in the shadow of the MFMAs)
    constexpr int UNITS = A_IT + B_IT, KS = BK / 16;
    auto compute = [&](int buf, auto stage_next, int buf_next) __attribute__((always_inline)) {
        const bf16_t* as = As + buf * A_BUF;
        const bf16_t* bs = Bs + buf * B_BUF;
        bf16x8 a[KS][TM], b[KS][TN];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = wm * TM * 32 + i * 32 + fidx;
                a[ks][i] = *reinterpret_cast<const bf16x8*>(as + row * LD + ks * 16 + kg * 8);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = wn * TN * 32 + j * 32 + fidx;
                b[ks][j] = *reinterpret_cast<const bf16x8*>(bs + row * LD + ks * 16 + kg * 8);
            }
        }
        [&]<int... KSI>(std::integer_sequence<int, KSI...>) {
            ([&] {
                constexpr int ks = KSI;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][i], b[ks][j], acc[i][j], 0, 0, 0);
                constexpr int u0 = ks * UNITS / KS, u1 = (ks + 1) * UNITS / KS;
                if constexpr (u1 > u0) {
                    __builtin_amdgcn_sched_barrier(0);
                    [&]<int... U>(std::integer_sequence<int, U...>) {
                        (lstore_unit(stage_next, buf_next, std::integral_constant<int, u0 + U>()), ...);
                    }(std::make_integer_sequence<int, u1 - u0>());
                    __builtin_amdgcn_sched_barrier(0);
                }
            }(), ...);
        }(std::make_integer_sequence<int, KS>());
        if constexpr (EP::kColSum) {          // bias gradient: sums of the B tile's rows (a row holds one column's k)
            if (c_tile % m_tiles == 0 && tid >= CS0 && tid - CS0 < BN) {
#pragma unroll
                for (int c = 0; c < BK / 8; ++c) {
                    const uint4 v = *reinterpret_cast<const uint4*>(bs + (tid - CS0) * LD + c * 8);
                    colsum = dot2_ones(v.w, dot2_ones(v.z, dot2_ones(v.y, dot2_ones(v.x, colsum))));
                }
            }
        }
    };
    // Epilogues with a bf16 output tile (kEntry): the finished tile goes through LDS and leaves as
    // 16-byte stores, 8 consecutive columns per thread, instead of 2-byte stores straight from the
    // accumulator layout (one eighth of the global memory instructions; the ReLU mask is read with
    // 16-byte loads as well).  Addresses and mask are fetched right after the tile's first barrier
    // (the row table is complete then) and arrive while the k loop runs.
    constexpr bool LOUT = EpiTraits<EP>::kEntry;
    constexpr int LDO = BN + 8, CPR = BN / 8, C_IT = LOUT ? BM * CPR / 256 : 1;
    static_assert(!LOUT || (BM * CPR) % 256 == 0, "whole chunks per thread");
    // the output tile reuses the operand buffers when it fits (the k loop ends with a barrier, and a
    // barrier after the tile's stores keeps the next tile's operands from overwriting it too early)
    constexpr bool OUT_ALIAS = LOUT && BM * LDO <= 2 * A_BUF + 2 * B_BUF;
    __shared__ __attribute__((aligned(16))) bf16_t outT_own[LOUT && !OUT_ALIAS ? BM * LDO : 8];
    bf16_t* const outT = OUT_ALIAS ? smem : outT_own;
    int cent[C_IT];
    uint4 caux[C_IT];
    float ebias[TN];
    auto tile_begin = [&]() __attribute__((always_inline)) {
        if constexpr (LOUT) {
            const int m0 = (c_tile % m_tiles) * BM, n0 = (c_tile / m_tiles) * BN;
#pragma unroll
            for (int c = 0; c < C_IT; ++c) {
                const int ch = tid + c * 256, lr = ch / CPR, c8 = ch % CPR;
                const int row = m0 + lr, col = n0 + c8 * 8;
                const bool ok = row < M && col < N;
                int base;
                if constexpr (EpiTraits<EP>::kRowTable) base = rowtab[tile_par * BM + lr];
                else base = ep.row_entry(ok ? row : 0, z);
                cent[c] = ok ? base + EpiColMap<EP>::off(ep, col) : -1;
                if constexpr (EP::kMask) caux[c] = *reinterpret_cast<const uint4*>(ep.mask() + (cent[c] >= 0 ? cent[c] : 0));
            }
            if constexpr (EP::kBias) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = n0 + wn * (TN * 32) + j * 32 + Mma<32>::col(lane);
                    ebias[j] = ep.bias[col < N ? col : 0];
                }
            }
        }
    };
    auto epilogue = [&]() __attribute__((always_inline)) {
        const int mt = c_tile % m_tiles, nt = c_tile / m_tiles;
        const int m0 = mt * BM, n0 = nt * BN;
        if constexpr (EP::kColSum) {
            if (mt == 0 && tid >= CS0 && tid - CS0 < BN && n0 + tid - CS0 < N) ep.store_colsum(n0 + tid - CS0, colsum, z);
            colsum = 0.f;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn * (TN * 32) + j * 32 + Mma<32>::col(lane);
                const bool full = m0 + BM <= M && n0 + BN <= N;     // interior tile (workgroup-uniform): no per-store test
                if constexpr (LOUT) {
                    const int lc = wn * (TN * 32) + j * 32 + Mma<32>::col(lane);
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int lr = wm * (TM * 32) + i * 32 + Mma<32>::row(r, lane);
                        outT[lr * LDO + lc] = ep.value(acc[i][j][r], EP::kBias ? ebias[j] : 0.f);
                    }
                } else {
                    typename EP::Aux aux[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = m0 + wm * (TM * 32) + i * 32 + Mma<32>::row(r, lane);
                        aux[r] = ep.aux(row, col, z, row < M && col < N);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = m0 + wm * (TM * 32) + i * 32 + Mma<32>::row(r, lane);
                        if (full || (row < M && col < N)) ep.store(row, col, acc[i][j][r], z, aux[r]);
                    }
                }
            }
        if constexpr (LOUT) {
            __syncthreads();
#pragma unroll
            for (int c = 0; c < C_IT; ++c) {
                const int ch = tid + c * 256, lr = ch / CPR, c8 = ch % CPR;
                uint4 v = *reinterpret_cast<const uint4*>(outT + lr * LDO + c8 * 8);
                if constexpr (EP::kMask) {
                    v.x = mask2(v.x, caux[c].x); v.y = mask2(v.y, caux[c].y); v.z = mask2(v.z, caux[c].z); v.w = mask2(v.w, caux[c].w);
                }
                if (cent[c] >= 0) *reinterpret_cast<uint4*>(ep.dst() + cent[c]) = v;
            }
            if constexpr (OUT_ALIAS) __syncthreads();
        }
        zero_acc();
    };
    auto step = [&](int kt, auto stage) __attribute__((always_inline)) {
        constexpr int G = decltype(stage)::value;
        constexpr int GN = (G + 1) % S;
        gload(kt + S, stage);
        if (ATAB && tid < BK) fill_tab(kt + S + 1, tid);          // read by the next step's gload, after this step's barrier
        compute(kt & 1, std::integral_constant<int, GN>(), (kt + 1) & 1);      // after the last k tile: zeros nobody reads
        __syncthreads();
    };
    for (; c_tile < tiles; c_tile += tile_stride, tile_par ^= 1) {
        set_load_tile(c_tile);
        if constexpr (EpiTraits<EP>::kRowTable) {
            static_assert(BM <= 256, "one thread per row of the tile");
            const int row = (c_tile % m_tiles) * BM + tid;
            if (tid < BM) rowtab[tile_par * BM + tid] = ep.row_entry(row < M ? row : 0, z);
        }
        if constexpr (ATAB) {
            for (int e = tid; e < RS * BK; e += 256) fill_tab(e / BK, e % BK);      // k tiles 0 .. S
            __syncthreads();
        }
        gload(0, std::integral_constant<int, 0>());
        gload(1, std::integral_constant<int, 1>());
        if constexpr (S > 2) gload(2, std::integral_constant<int, 2>());
        if constexpr (S > 3) gload(3, std::integral_constant<int, 3>());
        lstore(std::integral_constant<int, 0>(), 0);
        __syncthreads();
        tile_begin();
        // whole rounds of S steps without a branch, the remainder after the loop (see gemm_body)
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
        epilogue();          // the k loop ended with a barrier: the next tile may overwrite both LDS buffers
    }
}

// ----------------------------------------------------------------------------------------------
// RowK operands (contiguous along k)

// Addresses are split into a per-row byte offset (divisions, once per tile: Fixed) and a per-k byte
// offset; with lanes along the rows the latter is wave-uniform.  Out-of-range rows are clamped to row 0
// in Fixed and out-of-range k to 0, so every load is in bounds without per-lane address selects.
__device__ __forceinline__ const char* at(const void* base, int byte_off) {
    return static_cast<const char*>(base) + (unsigned)byte_off;      // tensors are far below 4 GiB
}

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

// ----------------------------------------------------------------------------------------------
// KRow operands (contiguous along m / n; var = reduction index)

template <class G> struct ConvNHWCKCols8 {     // A(m = (ky,kx,c), k = output position) from bf16 NHWC
    static constexpr bool kContig = false, kRowTab = true;
    typedef uint4 Raw;
    static __device__ __forceinline__ uint4 finish(Raw r, bool ok) { return keep_if_u4(ok, r); }
    const bf16_t* x; int rows;
    struct Fixed { int off; bool ok; };
    __device__ __forceinline__ Fixed prep(int col, int) const {
        Fixed f; f.ok = col < G::KK;
        col = f.ok ? col : 0;
        const int ky = col / (G::KS * G::CIN), rem = col % (G::KS * G::CIN);
        f.off = (ky * (G::W * G::CIN) + rem) * 2;
        return f;
    }
    __device__ __forceinline__ int row_entry(int row) const {
        if (row >= rows) return -1;
        const int n = row / (G::HO * G::WO), r = row % (G::HO * G::WO), oy = r / G::WO, ox = r % G::WO;
        return (((n * G::H + oy * G::ST) * G::W + ox * G::ST) * G::CIN) * 2;
    }
    __device__ __forceinline__ Raw load_at(const Fixed& f, int ent, bool pred, bool& ok) const {
        ok = pred && f.ok && ent >= 0;
        return *reinterpret_cast<const uint4*>(at(x, ok ? ent + f.off : 0));
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
struct EpiDenseMaskB {          // out[row][col] = v * 1[act[row][col] > 0]
    static constexpr bool kColSum = false, kEntry = true, kRowTable = false, kMask = true, kBias = false;
    bf16_t* out; const bf16_t* act; int ld; const float* bias;
    __device__ __forceinline__ int row_entry(int row, int) const { return row * ld; }
    __device__ __forceinline__ bf16_t value(float v, float) const { return f2bf(v); }
    __device__ __forceinline__ bf16_t* dst() const { return out; }
    __device__ __forceinline__ const bf16_t* mask() const { return act; }
};

// Grid: every k-split (grid y) gets min(tiles, resident workgroups of the whole chip) workgroups.
template <class T, class AL, class BL, class EP>
inline hipError_t launch_gemm_bf16(hipStream_t s, const AL& al, const BL& bl, const EP& ep, int M, int N, int K,
                                   int z_count, int k_per_split, int group_m = 0) {
    const int m_tiles = (M + T::BM - 1) / T::BM, n_tiles = (N + T::BN - 1) / T::BN;
    if (M <= 0 || N <= 0 || z_count <= 0) return hipErrorInvalidValue;
    const int tiles = m_tiles * n_tiles;
    if (group_m > 0) {              // XCD-grouped, one tile per workgroup (see the kernel)
        if (m_tiles % group_m != 0) return hipErrorInvalidValue;
        const int groups = (m_tiles / group_m) * z_count, gsz = group_m * n_tiles;
        launch_k((gemm_bf16_kernel<T, AL, BL, EP>), dim3(8 * ((groups + 7) / 8) * gsz, 1, 1), dim3(256), s, al, bl, ep, M, N, K,
                 k_per_split, m_tiles, n_tiles, group_m, z_count);
        return hipGetLastError();
    }
    static int resident = 0;           // workgroups of this kernel the device holds at once
    if (resident == 0) {
        int per_cu = 0, dev = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemm_bf16_kernel<T, AL, BL, EP>, 256, 0) != hipSuccess || per_cu < 1) per_cu = 1;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        resident = per_cu * cus;
    }
    // a grid up to a few times the resident set is started whole (its tail balances better than a
    // second full round of a persistent grid); beyond that the grid is the resident set
    const int gx = (tiles * z_count <= 4 * resident) ? tiles : std::max(1, resident / z_count);
    launch_k((gemm_bf16_kernel<T, AL, BL, EP>), dim3(gx, z_count, 1), dim3(256), s, al, bl, ep, M, N, K,
             k_per_split, m_tiles, n_tiles, 0, z_count);
    return hipGetLastError();
}

}  // namespace paac
