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

// Tile choice: rows by M (output channels are often 32..128), columns 128 unless N is tiny.
template <template <int> class AL, template <int> class BL, class Epi, class AP, class BP>
hipError_t launch_gemm(const AP &pa, const BP &pb, const typename Epi::Params &pe, const GemmShape &g,
                       hipStream_t s)
{
    const bool narrow = g.N <= 64;
    if (g.M <= 32) {
        return launch_tile<Tile<32, 128, 1, 4>, AL, BL, Epi>(pa, pb, pe, g, s);
    } else if (g.M <= 64 || (g.M % 128 != 0 && g.M % 128 <= 64 && g.M < 256)) {
        if (narrow) return launch_tile<Tile<64, 64, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
        return launch_tile<Tile<64, 128, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
    } else {
        if (narrow) return launch_tile<Tile<128, 64, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
        return launch_tile<Tile<128, 128, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
    }
}

}  // namespace ucd
