// Host-side tile choice and launch of gemm_kernel.
#pragma once
#include <string>

#include "gemm_core.hpp"
#include "kernels.h"

namespace ucd {

struct GemmShape {
    int M, N, Kd;
    int splits = 1;   // reduction splits (epilogue must accumulate when > 1)
    int batch = 1;    // independent GEMMs, operands advanced by the strides below
    long a_batch = 0, b_batch = 0, c_batch = 0;
    bool tail_split = false;  // the epilogue may split the tiles of a nearly empty last round
};

// Compute units of the current device (256 on a whole MI355X; fewer in a partitioned mode).  The
// launch heuristics fill rounds of this many workgroups.  Without a device (host-only planning,
// launch descriptions) the MI355X's count is assumed.
inline int device_cus()
{
    constexpr int kDefault = 256, kMaxDevices = 64;
    static int cached[kMaxDevices];   // 0 = not asked yet; a racing first call writes the same value
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return kDefault;
    }
    int v = cached[dev];
    if (v == 0) {
        v = kDefault;
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) v = n;
        else (void)hipGetLastError();
        cached[dev] = v;
    }
    return v;
}
constexpr int kTailMinSteps = 8;    // a tail workgroup's run has at least this many reduction steps (of BK rows)
constexpr int kTailMaxTiles = 224;  // a last round fuller than this is left alone

// Reduction chunks are whole steps of BK rows: the chunk length for a requested split count, and the
// number of chunks that really results.
inline int effective_splits(int Kd, int want, int &k_chunk)
{
    if (want < 1) want = 1;
    k_chunk = ((Kd + want - 1) / want + kBK - 1) / kBK * kBK;
    if (k_chunk < kBK) k_chunk = kBK;
    return Kd > 0 ? (Kd + k_chunk - 1) / k_chunk : 1;
}

template <class T, template <int> class AL, template <int> class BL, class Epi, class AP, class BP>
hipError_t launch_tile(const AP &pa, const BP &pb, const typename Epi::Params &pe, const GemmShape &g,
                       hipStream_t s)
{
    constexpr bool kVecLoads = vec_run<BL<T::BN>>(0);  // the bf16 kernel with vector operand loads
    // both operands bf16 tensors: the kernel on the bf16 matrix pipe (single GEMMs only)
    constexpr bool kBf16Mfma = AL<T::BM>::kBf16 && BL<T::BN>::kBf16;
    if (kBf16Mfma && g.batch != 1) return hipErrorInvalidValue;
    const int tiles_m = (g.M + T::BM - 1) / T::BM, tiles_n = (g.N + T::BN - 1) / T::BN;
    if (tiles_m <= 0 || tiles_n <= 0) return hipSuccess;
    int k_chunk;
    int splits = effective_splits(g.Kd, g.splits, k_chunk);
    if (kVecLoads) {  // that kernel's steps are kDeepBK rows
        k_chunk = (k_chunk + kDeepBK - 1) / kDeepBK * kDeepBK;
        splits = g.Kd > 0 ? (g.Kd + k_chunk - 1) / k_chunk : 1;
    }
    // Tail spreading (see TailSplit): when an unsplit GEMM's tile count is not a multiple of the CU
    // count, the reduction steps of the tiles beyond the last multiple are dealt out evenly to (up to)
    // one workgroup per CU, so that every CU gets the same work.
    TailSplit tail{0, 1, 0};
    if constexpr (Epi::kCanAdd) {
        const long tiles = (long)tiles_m * tiles_n;
        const int kCUs = device_cus();
        const int over = (int)(tiles % kCUs);
        if (g.tail_split && splits == 1 && g.batch == 1 && tiles >= 2 * kCUs && over > 0 && over <= kTailMaxTiles * kCUs / 256) {
            const int ksteps = (g.Kd + kBK - 1) / kBK;
            const long steps = (long)over * ksteps;
            long wgs = steps / kTailMinSteps;
            if (wgs > kCUs) wgs = kCUs;
            if (wgs > over && steps < (1l << 30)) {   // more workgroups than tiles, or nothing is gained
                tail.tiles = over;
                tail.wgs = (int)wgs;
                tail.ksteps = ksteps;
            }
        }
    }
    const unsigned gx = (unsigned)(tiles_m * tiles_n - tail.tiles + (tail.tiles ? tail.wgs : 0));
    dim3 grid(gx, (unsigned)splits, (unsigned)g.batch);
    if (LaunchLog *log = launch_log()) {
        if (tail.tiles) log->add("zero_tiles_kernel");
        log->add(std::string(kVecLoads ? "gemm_kernel_bf16v<Tile<" : kBf16Mfma ? "gemm_kernel_bf16<Tile<" : "gemm_kernel<Tile<") + std::to_string(T::BM) + "x" + std::to_string(T::BN) + ">," +
                 AL<T::BM>::name() + "," + BL<T::BN>::name() + "," + Epi::name() + "> tiles=" +
                 std::to_string(tiles_m * tiles_n) + " splits=" + std::to_string(splits) + " batch=" +
                 std::to_string(g.batch) + " M=" + std::to_string(g.M) + " N=" + std::to_string(g.N) + " K=" +
                 std::to_string(g.Kd) +
                 (tail.tiles ? " tail=" + std::to_string(tail.tiles) + "/" + std::to_string(tail.wgs) : std::string()));
        return hipSuccess;
    }
    if (tail.tiles) {
        zero_tiles_kernel<T, Epi><<<(unsigned)tail.tiles, kThreads, 0, s>>>(pe, g.M, g.N, tiles_m, tiles_n, tail.tiles);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if constexpr (kVecLoads)
        gemm_kernel_bf16v<T, AL<T::BM>, BL<T::BN>, Epi, AP, BP><<<grid, kThreads, 0, s>>>(
            pa, pb, pe, g.M, g.N, g.Kd, k_chunk, tiles_m, tiles_n);
    else if constexpr (kBf16Mfma)
        gemm_kernel_bf16<T, AL<T::BM>, BL<T::BN>, Epi, AP, BP><<<grid, kThreads, 0, s>>>(
            pa, pb, pe, g.M, g.N, g.Kd, k_chunk, tiles_m, tiles_n);
    else
        gemm_kernel<T, AL<T::BM>, BL<T::BN>, Epi, AP, BP><<<grid, kThreads, 0, s>>>(
            pa, pb, pe, g.M, g.N, g.Kd, k_chunk, tiles_m, tiles_n, g.a_batch, g.b_batch, g.c_batch, tail);
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

// Tile for a GEMM that will run `mult` times in one launch (reduction splits x batch): rows as
// above, 128 columns unless N is tiny; when that leaves the launch with fewer workgroups than CUs,
// narrower and then shorter tiles are taken to put more workgroups on the chip.
struct TilePick {
    int bm, bn;
    long blocks(int M, int N, long mult) const { return (long)((M + bm - 1) / bm) * ((N + bn - 1) / bn) * mult; }
};
inline TilePick pick_tile(int M, int N, bool rows96, long mult)
{
    // 64 columns when that wastes enough fewer padded columns to pay for the narrower tile's
    // lower MFMA-per-load ratio (N = 147: 192 columns instead of 256)
    const long pad128 = (long)(N + 127) / 128 * 128, pad64 = (long)(N + 63) / 64 * 64;
    TilePick t{pick_rows(M, rows96), (double)pad64 * 1.10 < (double)pad128 ? 64 : 128};
    if (t.bm == 32 || t.bm == 96) return t;  // single shapes
    if (t.blocks(M, N, mult) < 256 && t.bn == 128) t.bn = 64;
    if (t.blocks(M, N, mult) < 256 && t.bm == 128) t.bm = 64;
    return t;
}

template <template <int> class AL, template <int> class BL, class Epi, bool ROWS96 = false, class AP, class BP>
hipError_t launch_gemm(const AP &pa, const BP &pb, const typename Epi::Params &pe, const GemmShape &g,
                       hipStream_t s)
{
    const TilePick t = pick_tile(g.M, g.N, ROWS96, (long)(g.splits < 1 ? 1 : g.splits) * g.batch);
    if (t.bm == 32) return launch_tile<Tile<32, 128, 1, 4>, AL, BL, Epi>(pa, pb, pe, g, s);
    if (t.bm == 64) {
        if (t.bn == 64) return launch_tile<Tile<64, 64, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
        return launch_tile<Tile<64, 128, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
    }
    if constexpr (ROWS96) {
        if (t.bm == 96) return launch_tile<Tile<96, 128, 1, 4>, AL, BL, Epi>(pa, pb, pe, g, s);
    }
    if (t.bn == 64) return launch_tile<Tile<128, 64, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
    return launch_tile<Tile<128, 128, 2, 2>, AL, BL, Epi>(pa, pb, pe, g, s);
}

}  // namespace ucd
