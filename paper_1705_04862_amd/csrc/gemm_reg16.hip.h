// 16 x 16 output tiles straight from global memory into MFMA operand registers, for the launches of
// action selection at a batch of a few dozen states (Algorithm 1, the forward pass that evaluates
// pi(.|s; theta) for all n_e environments at once).
//
// At that size a GEMM of the network is a few hundred workgroups and each one ends before the machine
// has even been filled: its time is one chain of latencies.  The staged kernel of gemm_core.hip.h pays a
// chain per k-tile (global load -> LDS store -> barrier -> LDS read -> MFMA); here a workgroup has no k
// loop at all.  Its KW wavefronts divide the reduction range between them, every wavefront issues all
// the loads of its share at once in the register layout of the 16x16x4 MFMA, multiplies as they arrive,
// and the KW accumulators are added through LDS: one global round trip, one barrier.
//
// Operand A comes through the row-major loader interface of gemm_core.hip.h (four consecutive k per
// lane), operand B is a row-major (k, n) matrix read with one 4-byte load per k: sixteen lanes read
// sixteen consecutive columns, 64 contiguous bytes.
#pragma once
#include "gemm_core.hip.h"

namespace paac {

// A workgroup computes 16 rows x TN column fragments of 16 (the A registers serve all TN).
// KW wavefronts; a wavefront takes NG groups of 16 consecutive k per round (one round covers
// KW * NG * 16 values of k; more rounds follow while the split's range lasts).
template <int KW, int NG, int TN, class AL, class EP>
__global__ __launch_bounds__(KW * 64) void gemm_reg16_kernel(const AL al, const DenseKCols bl, const EP ep, int M, int N,
                                                             int K, int k_per_split, int m_tiles, int n_fast) {
    typedef Mma<16> MM;
    static_assert(AL::kContig, "operand A is read along k");
    static_assert(!EP::kColSum && !SplitAddr<EP>::value, "plain epilogues only");
    __shared__ __attribute__((aligned(16))) float red[(KW - 1) * TN * 64 * 4];

    int id = blockIdx.x + gridDim.x * blockIdx.y;
    id = xcd_order(id, gridDim.x * gridDim.y);
    const int tile = id % (int)gridDim.x, z = id / (int)gridDim.x;
    // Neighbours in the tile order run on one XCD and share its L2: they should share the larger operand.
    // With more row tiles than column tiles that is A (n_fast: the column tiles of one row tile are
    // neighbours), else B.  Measured at n_e = 32 on the second layer of arch_nature (162 x 4 tiles):
    // 6.95 -> 6.73 us, and the launch after it starts earlier (the whole selection call 28.6 -> 27.4 us).
    const int n_tiles = (int)gridDim.x / m_tiles;
    const int m0 = (n_fast ? tile / n_tiles : tile % m_tiles) * 16, n0 = (n_fast ? tile % n_tiles : tile / m_tiles) * (16 * TN);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int fidx = lane & 15, fk = lane >> 4;
    const int k_begin = k_per_split > 0 ? z * k_per_split : 0;
    const int k_end = k_per_split > 0 ? min(K, k_begin + k_per_split) : K;

    // accumulator register r of this lane is C[m0 + 4 fk + r][n0 + fidx]
    const int out_col = n0 + fidx;                  // + 16 t for column fragment t
    typename EP::Aux aux[TN][MM::NACC];
    auto load_aux = [&]() {
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int r = 0; r < MM::NACC; ++r) {
                const int row = m0 + MM::row(r, lane);
                aux[t][r] = ep.aux(row, out_col + 16 * t, z, wave == 0 && row < M && out_col + 16 * t < N);
            }
    };
    if constexpr (AuxEarly<EP>::value) load_aux();

    const typename AL::Fixed af = al.prep(m0 + fidx, z);
    const float* bp[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t) bp[t] = bl.base + (out_col + 16 * t < bl.cols ? out_col + 16 * t : 0);

    typename MM::Acc acc[TN][2];
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int r = 0; r < MM::NACC; ++r) acc[t][q][r] = 0.f;

    // MFMA step j of a group multiplies k = group start + 4 fk + j in lane group fk (both operands use the
    // same order, so any assignment of k to steps is a valid dot product)
    for (int base = k_begin + wave * (NG * 16); base < k_end; base += KW * NG * 16) {
        typename AL::Raw a[NG];
        float b[NG][TN][4];
        bool ok[NG];
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const int k = base + i * 16 + 4 * fk;
            const bool in = k < k_end;
            a[i] = al.load(af, k, in, ok[i]);
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                const float* q = bp[t] + (size_t)(in ? k : 0) * bl.ld;
#pragma unroll
                for (int j = 0; j < 4; ++j) b[i][t][j] = q[(size_t)j * bl.ld];
            }
        }
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            // rows past M and k past the end give zeros in A; B is read from a valid (clamped) address there
            const float4 v = AL::finish(a[i], ok[i]);
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                acc[t][0] = MM::mma(v.x, b[i][t][0], acc[t][0]);
                acc[t][1] = MM::mma(v.y, b[i][t][1], acc[t][1]);
                acc[t][0] = MM::mma(v.z, b[i][t][2], acc[t][0]);
                acc[t][1] = MM::mma(v.w, b[i][t][3], acc[t][1]);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int r = 0; r < MM::NACC; ++r) acc[t][0][r] += acc[t][1][r];

    if (wave > 0) {
#pragma unroll
        for (int t = 0; t < TN; ++t) *reinterpret_cast<f32x4*>(red + (((wave - 1) * TN + t) * 64 + lane) * 4) = acc[t][0];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int q = 0; q < KW - 1; ++q)
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(red + ((q * TN + t) * 64 + lane) * 4);
#pragma unroll
            for (int r = 0; r < MM::NACC; ++r) acc[t][0][r] += v[r];
        }
    if constexpr (!AuxEarly<EP>::value) load_aux();
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int r = 0; r < MM::NACC; ++r) {
            const int row = m0 + MM::row(r, lane);
            if (row < M && out_col + 16 * t < N) ep.store(row, out_col + 16 * t, acc[t][0][r], z, aux[t][r]);
        }
}

// Requirements checked here: every k range starts at a multiple of 4 (the loaders read 16 bytes) and the
// 4 k of a lane never straddle the end of a range, i.e. K and k_per_split are multiples of 4.
template <int TN = 1, class AL, class EP>
inline hipError_t launch_gemm_reg16(hipStream_t s, const AL& al, const DenseKCols& bl, const EP& ep, int M, int N, int K,
                                    int z_count, int k_per_split) {
    constexpr int KW = 8;       // four wavefronts (twice the chain of MFMAs each) measured slower: 6.95 -> 7.32 us
    if (M <= 0 || N <= 0 || z_count <= 0 || K % 4 != 0 || k_per_split % 4 != 0) return hipErrorInvalidValue;
    const int m_tiles = (M + 15) / 16, n_tiles = (N + 16 * TN - 1) / (16 * TN);
    const int range = k_per_split > 0 ? (k_per_split < K ? k_per_split : K) : K;
    const int groups_per_wave = ((range + 15) / 16 + KW - 1) / KW;
    const dim3 grid(m_tiles * n_tiles, z_count, 1), block(KW * 64);
    const int n_fast = m_tiles > n_tiles;
    if (groups_per_wave <= 2) launch_k((gemm_reg16_kernel<KW, 2, TN, AL, EP>), grid, block, s, al, bl, ep, M, N, K, k_per_split, m_tiles, n_fast);
    else if (groups_per_wave <= 4) launch_k((gemm_reg16_kernel<KW, 4, TN, AL, EP>), grid, block, s, al, bl, ep, M, N, K, k_per_split, m_tiles, n_fast);
    else launch_k((gemm_reg16_kernel<KW, 5, TN, AL, EP>), grid, block, s, al, bl, ep, M, N, K, k_per_split, m_tiles, n_fast);
    return hipGetLastError();
}

}  // namespace paac
