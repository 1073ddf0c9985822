// Zero-workspace implicit-GEMM convolution: Forward, BackwardData, BackwardFilter as tile GEMMs
// whose operand loaders gather straight from the NCHW tensors.
//   Forward        Y[K x bPQ]   = W[K x CRS]      * im2col(X)[CRS x bPQ]
//   BackwardData   dX[C x bHW]  = W^T[C x KRS]    * gather(dY)[KRS x bHW]   (one GEMM per stride phase)
//   BackwardFilter dW[K x CRS] += dY[K x bPQ]     * im2col(X)^T[bPQ x CRS]  (split over bPQ, fp32 atomics)
#include <cstdlib>
#include <type_traits>

#include "gemm_launch.hpp"
#include "kernels.h"

namespace ucd {

__global__ void fill_zero_kernel(float *p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += step) p[i] = 0.f;
}

LaunchLog *&launch_log()
{
    static thread_local LaunchLog *log = nullptr;
    return log;
}

hipError_t fill_zero(float *p, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    if (LaunchLog *log = launch_log()) {
        log->add("fill_zero_kernel");
        return hipSuccess;
    }
    size_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    fill_zero_kernel<<<(unsigned)blocks, 256, 0, s>>>(p, n);
    return hipGetLastError();
}

// A CU holds several of these workgroups at once (four of the Forward / BackwardData kernels,
// three of the BackwardFilter ones, by registers and LDS) and needs them all to keep its matrix
// pipes busy; workgroups of one launch take equally long, so a launch proceeds in rounds of
// 256 x resident workgroups, and a last round that is nearly empty costs as much as a full one
// (measured: the time of a Forward launch is flat from 769 to 1024 tiles).  Split counts are
// chosen so that the workgroup count fills its rounds.
static long slots_output() { return 4l * device_cus(); }
static long slots_filter() { return 3l * device_cus(); }

static double round_fill(long blocks, long slots)
{
    return (double)blocks / (double)((blocks + slots - 1) / slots * slots);
}

// Among split counts in [lo, hi], the one whose workgroup count fills its rounds best (ties: the
// one nearest to `want`).
static int best_fill(long tiles, long want, long lo, long hi, long slots)
{
    if (lo < 1) lo = 1;
    if (hi < lo) hi = lo;
    long best = want < lo ? lo : (want > hi ? hi : want);
    double best_f = round_fill(tiles * best, slots);
    for (long c = lo; c <= hi; ++c) {
        const double f = round_fill(tiles * c, slots);
        const long dc = c > want ? c - want : want - c, db = best > want ? best - want : want - best;
        if (f > best_f + 1e-9 || (f > best_f - 1e-9 && dc < db)) { best = c; best_f = f; }
    }
    return (int)best;
}

// Forward / BackwardData write each output once, so normally one workgroup owns a whole
// reduction.  When the output has too few tiles to give every CU several workgroups (deep
// layers: many channels, few pixels), the reduction is split as well and the partial results meet
// through atomics in a zero-filled output.  Chunks keep at least 512 reduction rows.
static int output_splits(int M, int N, int Kd, bool fp32_out)
{
    if (!fp32_out) return 1;  // bf16 outputs cannot be accumulated with atomics (nor may reproducible runs)
    const long tiles = pick_tile(M, N, true, 1 << 20).blocks(M, N, 1);  // tiles at the default shape
    if (tiles >= 768) return 1;  // three workgroups per CU already
    long want = (1536 + tiles - 1) / tiles;
    const long cap = Kd / 512;
    if (want > cap) want = cap;
    if (want < 2) return 1;
    return best_fill(tiles, want, want / 2 < 2 ? 2 : want / 2, want * 2 < cap ? want * 2 : cap, slots_output());
}

// bf16 tensors, stride-1 layers whose output rows are as wide as the input rows (so that, for every
// tap, neighbouring pixels of an image are neighbours in memory), filters of at most 31 taps: the
// activation operand is fetched four pixels per load (RunNLaneT).  Tile positions run over the
// images with their pixel count rounded up to 4.
static bool vector_gather_applies(const Dims &d, int grid_w, int tensor_w)
{
    // UCD_BF16_ELEMENTWISE=1 keeps the element-wise kernel (for comparisons)
    static const bool off = [] { const char *e = std::getenv("UCD_BF16_ELEMENTWISE"); return e && e[0] == '1'; }();
    return !off && d.dtype == 1 && d.sh == 1 && d.sw == 1 && grid_w == tensor_w && d.R * d.S <= 31;
}

static hipError_t implicit_fwd_bf16_vec(const Dims &d, int b, const void *x, const void *w, void *y, hipStream_t s)
{
    const int px = d.P * d.Q, px_pad = (px + 3) / 4 * 4;
    GemmShape g{d.K, b * px_pad, d.crs()};
    RunParams pb{};
    pb.t = x; pb.bytes = xbytes(d, b); pb.Ct = d.C; pb.Ht = d.H; pb.Wt = d.W;
    pb.plane_px = px; pb.grid_pad = FastDiv(px_pad); pb.grid_w = FastDiv(d.Q);
    pb.add_h = -d.ph; pb.add_w = -d.pw; pb.dir = 1;
    pb.taps = FastDiv(d.R * d.S); pb.taps_w = FastDiv(d.S);
    pb.n_tap_h = d.R; pb.n_tap_w = d.S;
    pb.shift_thread = d.ph * d.W + d.pw; pb.shift_row = 0;
    EpiNCHWParams pe{};
    pe.out = y; pe.grid_hw = pb.grid_pad; pe.grid_w = pb.grid_w;
    pe.M = d.K; pe.HWo = px; pe.Wo = d.Q; pe.h0 = 0; pe.hs = 1; pe.w0 = 0; pe.ws = 1; pe.cols = px;
    // 0: every element exists (no border masks); 1: masks, at most 16 taps; 2: masks, more taps
    const int mode = d.R * d.S == 1 && d.ph == 0 && d.pw == 0 ? 0 : d.R * d.S <= 16 ? 1 : 2;
    if (d.crs() % 8 == 0) {  // filter rows are whole 16-byte cells
        CellParams pa{w, wbytes(d), d.crs()};
        if (mode == 0) return launch_gemm<CellKLaneT, RunNLane, EpiNCHWT<bf16>, true>(pa, pb, pe, g, s);
        if (mode == 1) return launch_gemm<CellKLaneT, RunNLaneMasked, EpiNCHWT<bf16>, true>(pa, pb, pe, g, s);
        return launch_gemm<CellKLaneT, RunNLaneMaskedBig, EpiNCHWT<bf16>, true>(pa, pb, pe, g, s);
    }
    KLaneParams pa{};
    pa.t = w; pa.bytes = wbytes(d); pa.row_stride = 1; pa.col_stride = d.crs();
    if (mode == 0) return launch_gemm<Loaders<bf16>::KLane0, RunNLane, EpiNCHWT<bf16>, true>(pa, pb, pe, g, s);
    if (mode == 1) return launch_gemm<Loaders<bf16>::KLane0, RunNLaneMasked, EpiNCHWT<bf16>, true>(pa, pb, pe, g, s);
    return launch_gemm<Loaders<bf16>::KLane0, RunNLaneMaskedBig, EpiNCHWT<bf16>, true>(pa, pb, pe, g, s);
}

template <class E>
static hipError_t implicit_fwd_t(const Dims &d, int b, const void *x, const void *w, void *y, hipStream_t s)
{
    typedef Loaders<E> L;
    constexpr bool F32 = std::is_same<E, float>::value;
    if constexpr (!F32) {
        if (vector_gather_applies(d, d.Q, d.W)) return implicit_fwd_bf16_vec(d, b, x, w, y, s);
    }
    GemmShape g{d.K, b * d.P * d.Q, d.crs()};
    g.splits = output_splits(g.M, g.N, g.Kd, F32 && !d.det);
    KLaneParams pa{};
    pa.t = w; pa.bytes = wbytes(d); pa.row_stride = 1; pa.col_stride = d.crs();
    GatherParams pb{};
    pb.t = x; pb.bytes = xbytes(d, b); pb.Ct = d.C; pb.Ht = d.H; pb.Wt = d.W;
    pb.grid_hw = FastDiv(d.P * d.Q); pb.grid_w = FastDiv(d.Q);
    pb.mul_h = d.sh; pb.add_h = -d.ph; pb.mul_w = d.sw; pb.add_w = -d.pw; pb.dir = 1;
    pb.taps = FastDiv(d.R * d.S); pb.taps_w = FastDiv(d.S);
    pb.n_tap_h = d.R; pb.n_tap_w = d.S;
    pb.shift_thread = d.ph * d.W + d.pw; pb.shift_row = 0;
    EpiNCHWParams pe{};
    pe.out = y; pe.grid_hw = pb.grid_hw; pe.grid_w = pb.grid_w;
    pe.M = d.K; pe.HWo = d.P * d.Q; pe.Wo = d.Q; pe.h0 = 0; pe.hs = 1; pe.w0 = 0; pe.ws = 1;
    if constexpr (F32) {
        if (g.splits > 1) {
            hipError_t e = fill_zero((float *)y, (size_t)b * d.K * d.P * d.Q, s);
            if (e != hipSuccess) return e;
            if (d.R * d.S <= 31) return launch_gemm<KLane0, GatherNLane, EpiNCHWAtomic, true>(pa, pb, pe, g, s);
            return launch_gemm<KLane0, GatherNLaneBig, EpiNCHWAtomic, true>(pa, pb, pe, g, s);
        }
    }
    g.tail_split = !d.det;
    // without padding every tap of every output pixel lies inside x: the loader without border masks
    // (filters of more than one tap: 1x1 layers are bound by memory, not by the loader)
    if (d.ph == 0 && d.pw == 0 && d.R * d.S > 1)
        return launch_gemm<L::template KLane0, L::template GatherNLaneFree, EpiNCHWT<E>, true>(pa, pb, pe, g, s);
    if (d.R * d.S <= 31)
        return launch_gemm<L::template KLane0, L::template GatherNLane, EpiNCHWT<E>, true>(pa, pb, pe, g, s);
    return launch_gemm<L::template KLane0, L::template GatherNLaneBig, EpiNCHWT<E>, true>(pa, pb, pe, g, s);
}

hipError_t implicit_fwd(const Dims &d, int b, const void *x, const void *w, void *y, hipStream_t s)
{
    return d.dtype == 1 ? implicit_fwd_t<bf16>(d, b, x, w, y, s) : implicit_fwd_t<float>(d, b, x, w, y, s);
}

// Merged stride phases.  With few input channels a phase GEMM (M = C rows) leaves most of a
// 32-row tile empty.  Writing h + ph = vs*t + a with vs = f*stride, the pixels a = 0..vs-1 of
// block t are all reached from the same window of dy rows p = f*t + (f-1) - u, u = 0..U'-1,
// U' = ceil(R/stride) + f - 1, through filter row r = a - stride*(f-1) + stride*u (no such tap:
// zero).  One GEMM with M = C*vs_h*vs_w rows then computes all phases; R*S of every
// (stride*U')*(stride*V') taps it multiplies are real.  f = 1 or 2, whichever wastes least;
// 0 = keep the phases separate.
static int merged_phase_factor(const Dims &d)
{
    if (d.sh * d.sw == 1 || d.C >= 32) return 0;
    auto tile_eff = [](int M) {  // useful rows of the tiles x relative speed of the tile shape
        const int rows = pick_rows(M, true);
        const double speed = rows == 32 ? 0.7 : rows == 64 ? 0.9 : rows == 96 ? 0.96 : 1.0;
        return (double)M / ((M + rows - 1) / rows * rows) * speed;
    };
    int best = 0;
    double best_s = tile_eff(d.C);  // separate phases multiply no zero taps
    for (int f = 1; f <= 2; ++f) {
        const int M = d.C * f * d.sh * f * d.sw;
        const int U = (d.R + d.sh - 1) / d.sh + f - 1, V = (d.S + d.sw - 1) / d.sw + f - 1;
        if (M > 128 || U > 31 || V > 31) continue;
        const double s = tile_eff(M) * d.R / (double)(d.sh * U) * d.S / (double)(d.sw * V);
        if (s > best_s * 1.1) { best = f; best_s = s; }
    }
    return best;
}

template <class E>
static hipError_t implicit_bwd_data_merged(const Dims &d, int b, const void *dy, const void *w, void *dx, int f,
                                           hipStream_t s)
{
    typedef Loaders<E> L;
    const int vsh = f * d.sh, vsw = f * d.sw;
    const int U = (d.R + d.sh - 1) / d.sh + f - 1, V = (d.S + d.sw - 1) / d.sw + f - 1;
    const int Hb = (d.H - 1 + d.ph) / vsh + 1, Wb = (d.W - 1 + d.pw) / vsw + 1;  // blocks that hold a pixel
    GemmShape g{d.C * vsh * vsw, b * Hb * Wb, d.K * U * V};
    KLaneParams pa{};
    pa.t = w; pa.bytes = wbytes(d); pa.col_stride = d.R * d.S; pa.k_stride = d.crs(); pa.s_mem = d.S;
    pa.taps = FastDiv(U * V); pa.taps_w = FastDiv(V);
    pa.col_taps = FastDiv(vsh * vsw); pa.col_taps_w = FastDiv(vsw);
    pa.tap_mul_h = d.sh; pa.tap_add_h = -d.sh * (f - 1); pa.tap_mul_w = d.sw; pa.tap_add_w = -d.sw * (f - 1);
    pa.n_tap_h = d.R; pa.n_tap_w = d.S;
    GatherParams pb{};
    pb.t = dy; pb.bytes = ybytes(d, b); pb.Ct = d.K; pb.Ht = d.P; pb.Wt = d.Q;
    pb.grid_hw = FastDiv(Hb * Wb); pb.grid_w = FastDiv(Wb);
    pb.mul_h = f; pb.add_h = f - 1; pb.mul_w = f; pb.add_w = f - 1; pb.dir = -1;
    pb.taps = pa.taps; pb.taps_w = pa.taps_w;
    pb.n_tap_h = U; pb.n_tap_w = V;
    pb.shift_thread = 0; pb.shift_row = (U - 1) * d.Q + (V - 1);
    EpiPhasesParams pe{};
    pe.out = dx; pe.grid_hw = pb.grid_hw; pe.grid_w = pb.grid_w; pe.block = pa.col_taps; pe.block_w = pa.col_taps_w;
    pe.C = d.C; pe.H = d.H; pe.W = d.W; pe.vs_h = vsh; pe.vs_w = vsw; pe.pad_h = d.ph; pe.pad_w = d.pw;
    if (U * V <= 31)
        return launch_gemm<L::template PhaseFilterKLane, L::template GatherNLane, EpiPhasesT<E>, true>(pa, pb, pe, g, s);
    return launch_gemm<L::template PhaseFilterKLane, L::template GatherNLaneBig, EpiPhasesT<E>, true>(pa, pb, pe, g, s);
}

// One phase GEMM with the gather loader that fits its tap count.
template <template <int> class AL, template <int> class GatherSmall, template <int> class GatherBig, class Epi,
          bool ROWS96>
static hipError_t launch_phase(bool small, const KLaneParams &pa, const GatherParams &pb, const EpiNCHWParams &pe,
                               const GemmShape &g, hipStream_t s)
{
    return small ? launch_gemm<AL, GatherSmall, Epi, ROWS96>(pa, pb, pe, g, s)
                 : launch_gemm<AL, GatherBig, Epi, ROWS96>(pa, pb, pe, g, s);
}

// Stride-1 BackwardData with bf16 tensors and vector loads of dy (see vector_gather_applies): one
// GEMM dX[C x bHW] = W^T[C x KRS] * gather(dY), the gather running backwards through the taps.
static hipError_t implicit_bwd_data_bf16_vec(const Dims &d, int b, const void *dy, const void *w, void *dx,
                                             hipStream_t s)
{
    typedef Loaders<bf16> L;
    const int px = d.H * d.W, px_pad = (px + 3) / 4 * 4;
    GemmShape g{d.C, b * px_pad, d.K * d.R * d.S};
    KLaneParams pa{};
    pa.t = w; pa.bytes = wbytes(d); pa.col_stride = d.R * d.S;
    pa.taps = FastDiv(d.R * d.S); pa.taps_w = FastDiv(d.S);
    pa.k_stride = d.crs(); pa.s_mem = d.S;
    pa.tap_add_h = 0; pa.tap_mul_h = 1; pa.tap_add_w = 0; pa.tap_mul_w = 1;
    pa.unit_taps = 1;
    RunParams pb{};
    pb.t = dy; pb.bytes = ybytes(d, b); pb.Ct = d.K; pb.Ht = d.P; pb.Wt = d.Q;
    pb.plane_px = px; pb.grid_pad = FastDiv(px_pad); pb.grid_w = FastDiv(d.W);
    pb.add_h = d.ph; pb.add_w = d.pw; pb.dir = -1;
    pb.taps = pa.taps; pb.taps_w = pa.taps_w;
    pb.n_tap_h = d.R; pb.n_tap_w = d.S;
    pb.shift_thread = 0; pb.shift_row = (d.R - 1) * d.Q + (d.S - 1);
    EpiNCHWParams pe{};
    pe.out = dx; pe.grid_hw = pb.grid_pad; pe.grid_w = pb.grid_w;
    pe.M = d.C; pe.HWo = px; pe.Wo = d.W; pe.h0 = 0; pe.hs = 1; pe.w0 = 0; pe.ws = 1; pe.cols = px;
    const bool plain = d.R * d.S == 1 && d.ph == 0 && d.pw == 0;
    // filter operand: lanes along the input channels for filters of at most 9 taps (see below)
    if (pick_rows(d.C, true) != 96 && d.R * d.S <= 9)
        return plain ? launch_gemm<L::template FilterNLane, RunNLane, EpiNCHWT<bf16>, false>(pa, pb, pe, g, s)
                     : launch_gemm<L::template FilterNLane, RunNLaneMasked, EpiNCHWT<bf16>, false>(pa, pb, pe, g, s);
    return plain ? launch_gemm<L::template FilterKLane, RunNLane, EpiNCHWT<bf16>, true>(pa, pb, pe, g, s)
                 : launch_gemm<L::template FilterKLane, RunNLaneMaskedBig, EpiNCHWT<bf16>, true>(pa, pb, pe, g, s);
}

// Stride phases: input pixels h with (h + ph) % sh == a are reached only by filter rows
// r = a, a + sh, ...; within a phase the gather is a dense stride-1 correlation with the
// sub-sampled, index-reversed filter.  Pixels of a phase with no tap get zeros (Kd = 0).
template <class E>
static hipError_t implicit_bwd_data_t(const Dims &d, int b, const void *dy, const void *w, void *dx, hipStream_t s)
{
    typedef Loaders<E> L;
    constexpr bool F32 = std::is_same<E, float>::value;
    if constexpr (!F32) {
        // measured slower than the element-wise kernel (its filter operand cannot be fetched in cells
        // and, run four times per step, costs the kernel its second workgroup per CU): opt-in only
        static const bool on = [] { const char *e = std::getenv("UCD_BF16_VEC_BWD_DATA"); return e && e[0] == '1'; }();
        if (on && vector_gather_applies(d, d.W, d.Q)) return implicit_bwd_data_bf16_vec(d, b, dy, w, dx, s);
    }
    if (const int f = merged_phase_factor(d)) return implicit_bwd_data_merged<E>(d, b, dy, w, dx, f, s);
    // phases whose GEMM has too few tiles split their reduction (atomics); dx is zero-filled once
    // if any phase does
    auto phase_shape = [&](int a, int c, int &h0, int &w0, int &Hh, int &Ww, int &Ra, int &Sc) {
        h0 = ((a - d.ph) % d.sh + d.sh) % d.sh;
        w0 = ((c - d.pw) % d.sw + d.sw) % d.sw;
        Hh = h0 < d.H ? (d.H - h0 + d.sh - 1) / d.sh : 0;
        Ww = w0 < d.W ? (d.W - w0 + d.sw - 1) / d.sw : 0;
        Ra = a < d.R ? (d.R - a + d.sh - 1) / d.sh : 0;
        Sc = c < d.S ? (d.S - c + d.sw - 1) / d.sw : 0;
    };
    bool any_split = false;
    for (int a = 0; a < d.sh; ++a)
        for (int c = 0; c < d.sw; ++c) {
            int h0, w0, Hh, Ww, Ra, Sc;
            phase_shape(a, c, h0, w0, Hh, Ww, Ra, Sc);
            if (Hh && Ww && Ra && Sc && output_splits(d.C, b * Hh * Ww, d.K * Ra * Sc, F32 && !d.det) > 1) any_split = true;
        }
    if (any_split) {
        hipError_t e = fill_zero((float *)dx, (size_t)b * d.C * d.H * d.W, s);
        if (e != hipSuccess) return e;
    }
    for (int a = 0; a < d.sh; ++a)
        for (int c = 0; c < d.sw; ++c) {
            int h0, w0, Hh, Ww, Ra, Sc;
            phase_shape(a, c, h0, w0, Hh, Ww, Ra, Sc);
            if (Hh == 0 || Ww == 0) continue;
            GemmShape g{d.C, b * Hh * Ww, d.K * Ra * Sc};
            if (any_split && g.Kd == 0) continue;  // dx is already zero there
            g.splits = output_splits(g.M, g.N, g.Kd, F32 && !d.det);
            const bool split = g.splits > 1;
            KLaneParams pa{};
            pa.t = w; pa.bytes = wbytes(d); pa.col_stride = d.R * d.S;
            pa.taps = FastDiv(Ra * Sc); pa.taps_w = FastDiv(Sc);
            pa.k_stride = d.crs(); pa.s_mem = d.S;
            pa.tap_add_h = a; pa.tap_mul_h = d.sh; pa.tap_add_w = c; pa.tap_mul_w = d.sw;
            pa.unit_taps = (d.sh == 1 && d.sw == 1) ? 1 : 0;
            GatherParams pb{};
            pb.t = dy; pb.bytes = ybytes(d, b); pb.Ct = d.K; pb.Ht = d.P; pb.Wt = d.Q;
            pb.grid_hw = FastDiv(Hh * Ww); pb.grid_w = FastDiv(Ww);
            pb.mul_h = 1; pb.add_h = (h0 + d.ph - a) / d.sh; pb.mul_w = 1; pb.add_w = (w0 + d.pw - c) / d.sw;
            pb.dir = -1;
            pb.taps = pa.taps; pb.taps_w = pa.taps_w;
            pb.n_tap_h = Ra; pb.n_tap_w = Sc;
            pb.shift_thread = 0; pb.shift_row = (Ra > 0 ? Ra - 1 : 0) * d.Q + (Sc > 0 ? Sc - 1 : 0);
            EpiNCHWParams pe{};
            pe.out = dx; pe.grid_hw = pb.grid_hw; pe.grid_w = pb.grid_w;
            pe.M = d.C; pe.HWo = d.H * d.W; pe.Wo = d.W; pe.h0 = h0; pe.hs = d.sh; pe.w0 = w0; pe.ws = d.sw;
            // With 2-byte elements the filter operand is read with lanes along the input channels
            // instead of the reduction rows (FilterNLaneT: fewer cache accesses per load; AlexNet
            // conv4 at b = 256: 0.56 -> 0.44 ms), where the tile is not the one that loader lacks (96
            // rows) and the filter has at most 9 taps: its lanes are R*S elements apart, and
            // on a 5x5 filter it is the slower one by far (conv2: 0.76 -> 1.46 ms).  In fp32, where
            // vector and scalar instruction issue is the limit and not the memory pipeline, it
            // measured 5-10 % slower even on 1x1 filters, whose channels are contiguous in memory.
            const bool nlane = !F32 && pick_rows(d.C, true) != 96 && d.R * d.S <= 9;
            const bool small = Ra * Sc <= 31;
            hipError_t e = hipSuccess;
            bool done = false;
            if constexpr (F32) {
                if (split) {
                    e = launch_phase<FilterKLane, GatherNLane, GatherNLaneBig, EpiNCHWAtomic, true>(small, pa, pb, pe, g, s);
                    done = true;
                }
            }
            g.tail_split = !d.det;
            if constexpr (!F32) {
                if (nlane) {
                    e = launch_phase<L::template FilterNLane, L::template GatherNLane, L::template GatherNLaneBig,
                                     EpiNCHWT<E>, false>(small, pa, pb, pe, g, s);
                    done = true;
                }
            }
            if (!done)
                e = launch_phase<L::template FilterKLane, L::template GatherNLane, L::template GatherNLaneBig,
                                 EpiNCHWT<E>, true>(small, pa, pb, pe, g, s);
            if (e != hipSuccess) return e;
        }
    return hipSuccess;
}

hipError_t implicit_bwd_data(const Dims &d, int b, const void *dy, const void *w, void *dx, hipStream_t s)
{
    return d.dtype == 1 ? implicit_bwd_data_t<bf16>(d, b, dy, w, dx, s) : implicit_bwd_data_t<float>(d, b, dy, w, dx, s);
}

// ---- BackwardData on a mirrored filter copy ---------------------------------------------------------
// With stride 1, dx[n,c,h,w] = sum_{k,r,s} dy[n,k,h+pad-r,w+pad-s] w[k,c,r,s] is the Forward
// convolution of dy (K channels, P x Q) with wt[c][k][r'][s'] = w[k][c][R-1-r'][S-1-s'] and padding
// (R-1-pad, S-1-pad).  Once the filter is stored that way its rows are contiguous along the
// reduction index, which is what the Forward kernels' filter loaders want (no per-element decode
// in fp32; 16-byte cells for the bf16 vector-load kernel).  The copy costs K*C*R*S elements of
// workspace and one small kernel per run of micro-batches.
template <class E>
__global__ __launch_bounds__(256) void mirror_filter_kernel(const E *__restrict__ w, E *__restrict__ wt, int K, int C,
                                                            int RS)
{
    const long n = (long)K * C * RS;
    for (long i = blockIdx.x * 256l + threadIdx.x; i < n; i += 256l * gridDim.x) {
        const int t = (int)(i % RS);
        const long ck = i / RS;
        const int k = (int)(ck % K), c = (int)(ck / K);
        wt[i] = w[((long)k * C + c) * RS + (RS - 1 - t)];   // (R-1-r)*S + (S-1-s) = RS-1 - (r*S+s)
    }
}

bool implicit_mirror_applies(const Dims &d, int op)
{
    return op == 1 && d.sh == 1 && d.sw == 1 && d.ph <= d.R - 1 && d.pw <= d.S - 1;
}

size_t implicit_mirror_ws_bytes(const Dims &d) { return (d.esize() * d.K * d.crs() + 15) / 16 * 16; }

hipError_t implicit_bwd_data_mirror(const Dims &d, int b, const void *dy, const void *w, void *dx, void *ws,
                                    bool filter_ready, hipStream_t s)
{
    LaunchLog *log = launch_log();
    if (filter_ready) {
        // the copy is still in the workspace from the previous micro-batch
    } else if (log) {
        log->add("mirror_filter_kernel");
    } else {
        const long n = (long)d.K * d.crs();
        const unsigned blocks = (unsigned)((n + 255) / 256 < 2048 ? (n + 255) / 256 : 2048);
        if (d.dtype == 1)
            mirror_filter_kernel<uint16_t><<<blocks, 256, 0, s>>>((const uint16_t *)w, (uint16_t *)ws, d.K, d.C, d.R * d.S);
        else
            mirror_filter_kernel<float><<<blocks, 256, 0, s>>>((const float *)w, (float *)ws, d.K, d.C, d.R * d.S);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    Dims m = d;   // the mirrored layer: dy is its input, dx its output
    m.C = d.K; m.K = d.C;
    m.H = d.P; m.W = d.Q; m.P = d.H; m.Q = d.W;
    m.ph = d.R - 1 - d.ph; m.pw = d.S - 1 - d.pw;
    return implicit_fwd(m, b, dy, ws, dx, s);
}

// Number of reduction splits so that tiles * splits covers the chip a few times over, with
// chunks of at least 256 reduction rows.
int filter_splits(int M, int N, int Kd, int batch)
{
    const TilePick shape = pick_tile(M, N, true, 1 << 20);  // the default shape
    const long tiles = shape.blocks(M, N, batch);
    long want = (1024 + tiles - 1) / tiles;
    long cap = Kd / 256;
    if (cap < 1) cap = 1;
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    // three workgroups of the 96- and 128-row BackwardFilter kernels fit a CU, four of the others
    const long slots = shape.bm >= 96 ? slots_filter() : slots_output();
    if (tiles >= 4 * slots) return (int)want;  // many rounds anyway
    return best_fill(tiles, want, (want + 1) / 2, want * 2 < cap ? want * 2 : cap, slots);
}

// Reproducible BackwardFilter: at most this much workspace holds the reduction chunks' partial
// results (one K x CRS plane per chunk); a filter too large for several planes gets fewer, longer chunks.
constexpr size_t kDetPartialCap = (size_t)32 << 20;

static int det_filter_splits(const Dims &d, int b)
{
    const int Kd = b * d.P * d.Q;
    long want = filter_splits(d.K, d.crs(), Kd);
    const long cap = (long)(kDetPartialCap / ((size_t)4 * d.K * d.crs()));
    if (want > cap) want = cap;
    int chunk;
    return effective_splits(Kd, (int)(want < 1 ? 1 : want), chunk);
}

size_t implicit_det_ws_bytes(const Dims &d, int b)
{
    const int splits = det_filter_splits(d, b);
    return splits > 1 ? (size_t)4 * splits * d.K * d.crs() : 0;  // one chunk: a single addition per element
}

// dw = beta * dw + part[0] + part[1] + ... in that order
__global__ void reduce_partials_kernel(const float *part, int splits, size_t plane, float *dw, float beta, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += step) {
        float acc = beta == 0.f ? 0.f : dw[i];
        for (int sp = 0; sp < splits; ++sp) acc += part[(size_t)sp * plane + i];
        dw[i] = acc;
    }
}

template <class E>
static hipError_t implicit_bwd_filter_t(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                                        float *ws, hipStream_t s)
{
    typedef Loaders<E> L;
    hipError_t e;
    GemmShape g{d.K, d.crs(), b * d.P * d.Q};
    g.splits = d.det ? det_filter_splits(d, b) : filter_splits(g.M, g.N, g.Kd);
    const bool partials = d.det && g.splits > 1;
    if (!partials && beta == 0.f && (e = fill_zero(dw, (size_t)d.K * d.crs(), s)) != hipSuccess) return e;
    KLaneParams pa{};
    pa.t = dy; pa.bytes = ybytes(d, b);
    pa.grid_hw = FastDiv(d.P * d.Q); pa.grid_w = FastDiv(d.Q);
    pa.col_taps = FastDiv(1); pa.col_taps_w = FastDiv(1);
    pa.n_stride = d.K * d.P * d.Q; pa.Ht = d.P; pa.Wt = d.Q;
    pa.mul_h = 1; pa.add_h = 0; pa.mul_w = 1; pa.add_w = 0;
    KLaneParams pb{};
    pb.t = x; pb.bytes = xbytes(d, b);
    pb.grid_hw = pa.grid_hw; pb.grid_w = pa.grid_w;
    pb.col_taps = FastDiv(d.R * d.S); pb.col_taps_w = FastDiv(d.S);
    pb.n_stride = d.C * d.H * d.W; pb.Ht = d.H; pb.Wt = d.W;
    pb.mul_h = d.sh; pb.add_h = -d.ph; pb.mul_w = d.sw; pb.add_w = -d.pw;
    pb.shift = d.ph * d.W + d.pw;
    pb.n_tap_h = d.R; pb.n_tap_w = d.S;
    if (partials) {
        const size_t plane = (size_t)d.K * d.crs();
        EpiPartialParams pp{ws, d.crs(), (long)plane};
        if (d.R * d.S <= 31) e = launch_gemm<L::template DyTab, L::template XTab, EpiPartial, true>(pa, pb, pp, g, s);
        else e = launch_gemm<L::template DyKLane, L::template XKLane, EpiPartial, true>(pa, pb, pp, g, s);
        if (e != hipSuccess) return e;
        if (LaunchLog *log = launch_log()) {
            log->add("reduce_partials_kernel");
            return hipSuccess;
        }
        size_t blocks = (plane + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        reduce_partials_kernel<<<(unsigned)blocks, 256, 0, s>>>(ws, g.splits, plane, dw, beta, plane);
        return hipGetLastError();
    }
    EpiDenseParams pe{dw, d.crs()};
    if (d.R * d.S <= 31)  // per-row state in an LDS table
        return launch_gemm<L::template DyTab, L::template XTab, EpiAtomic, true>(pa, pb, pe, g, s);
    if (d.ph == 0 && d.pw == 0)  // no padding: every tap of every pixel is inside x
        return launch_gemm<L::template DyKLane, L::template XKLaneFree, EpiAtomic, true>(pa, pb, pe, g, s);
    return launch_gemm<L::template DyKLane, L::template XKLane, EpiAtomic, true>(pa, pb, pe, g, s);
}

hipError_t implicit_bwd_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                               float *ws, hipStream_t s)
{
    return d.dtype == 1 ? implicit_bwd_filter_t<bf16>(d, b, x, dy, dw, beta, ws, s)
                        : implicit_bwd_filter_t<float>(d, b, x, dy, dw, beta, ws, s);
}

}  // namespace ucd
