// Host-side tile choice and launch of gemm_kernel.
#pragma once
#include "gemm_core.hpp"

namespace ucd {

struct GemmShape {
    int M, N, Kd;
    int splits = 1;   // reduction splits (epilogue must accumulate when > 1)
    int batch = 1;    // independent GEMMs, operands advanced by the strides below
    long a_batch = 0, b_batch = 0, c_batch = 0;
};

template <class T, template <int> class AL, template <int> class BL, class Epi, class AP, class BP>
hipError_t launch_tile(const AP &pa, const BP &pb, const typename Epi::Params &pe, const GemmShape &g,
                       hipStream_t s)
{
    const int tiles_m = (g.M + T::BM - 1) / T::BM, tiles_n = (g.N + T::BN - 1) / T::BN;
    if (tiles_m <= 0 || tiles_n <= 0) return hipSuccess;
    int splits = g.splits < 1 ? 1 : g.splits;
    int k_chunk = ((g.Kd + splits - 1) / splits + kBK - 1) / kBK * kBK;
    if (k_chunk < kBK) k_chunk = kBK;
    splits = g.Kd > 0 ? (g.Kd + k_chunk - 1) / k_chunk : 1;
    dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)splits, (unsigned)g.batch);
    gemm_kernel<T, AL<T::BM>, BL<T::BN>, Epi, AP, BP><<<grid, kThreads, 0, s>>>(
        pa, pb, pe, g.M, g.N, g.Kd, k_chunk, tiles_m, tiles_n, g.a_batch, g.b_batch, g.c_batch);
    return hipGetLastError();
}

// Tile choice: 32 rows only for M <= 32; otherwise the row count among 128 / 96 / 64 with the
// least padded work, shorter tiles being charged for their lower MFMA-per-load ratio; 128 columns
// unless N is tiny.  96-row tiles (one wave column of three MFMA tiles) exist for the
// reduction-lane A loaders only (ROWS96): 96 channels are common (AlexNet's first two layers).
inline int pick_rows(int M, bool rows96)
{
    if (M <= 32) return 32;
    int best = 128;
    double best_cost = (double)((M + 127) / 128 * 128);
    const int cand[2] = {96, 64};
    const double charge[2] = {1.04, 1.10};
    for (int i = 0; i < 2; ++i) {
        if (cand[i] == 96 && !rows96) continue;
        const double cost = (double)((M + cand[i] - 1) / cand[i] * cand[i]) * charge[i];
        if (cost < best_cost) { best = cand[i]; best_cost = cost; }
    }
    return best;
}

template <template <int> class AL, template <int> class BL, class Epi, bool ROWS96 = false, class AP, class BP>
hipError_t launch_gemm(const AP &pa, const BP &pb, const typename Epi::Params &pe, const GemmShape &g,
                       hipStream_t s)
{
    const bool narrow = g.N <= 64;
    const int best = pick_rows(g.M, ROWS96);
    if (best == 32) return launch_tile<Tile<32, 128, 1, 4>, AL, BL, Epi>(pa, pb, pe, g, s);
    if (best == 64) {
        if (narrow) return launch_tile<Tile<64, 64, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
        return launch_tile<Tile<64, 128, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
    }
    if constexpr (ROWS96) {
        if (best == 96) return launch_tile<Tile<96, 128, 1, 4>, AL, BL, Epi>(pa, pb, pe, g, s);
    }
    if (narrow) return launch_tile<Tile<128, 64, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
    return launch_tile<Tile<128, 128, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
}

}  // namespace ucd
