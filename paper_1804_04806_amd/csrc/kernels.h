// Host-side launchers of the HIP kernels.  Every launcher only enqueues on `stream` and returns
// the launch status; pointers are device pointers already offset to the micro-batch.
#pragma once
#include <hip/hip_runtime.h>
#include <cstddef>
#include <cstdint>
#include <string>

namespace ucd {

// dtype 0: every tensor fp32.  dtype 1: x, w, dy, y, dx are bf16; dw and every workspace matrix
// stay fp32, accumulation is fp32 everywhere.
struct Dims {
    int C, H, W, K, R, S, sh, sw, ph, pw, P, Q;
    int dtype;
    // Reproducible mode: no launch accumulates with atomics in an order that can change from run to
    // run.  Forward / BackwardData never split their reductions; BackwardFilter (implicit GEMM only)
    // keeps its reduction chunks' partial results in workspace and sums them in a fixed order.
    bool det;
    int crs() const { return C * R * S; }
    size_t esize() const { return dtype == 1 ? 2 : 4; }
};

// operand sizes in bytes (each at most 2 GiB, checked before any launch)
inline uint32_t wbytes(const Dims &d) { return (uint32_t)(d.esize() * d.K * d.crs()); }
inline uint32_t xbytes(const Dims &d, int b) { return (uint32_t)(d.esize() * b * d.C * d.H * d.W); }
inline uint32_t ybytes(const Dims &d, int b) { return (uint32_t)(d.esize() * b * d.K * d.P * d.Q); }

// Winograd F(2x2,5x5) with fused transforms: Forward / BackwardData of 5x5 stride-1 layers with
// horizontal padding 2, fp32 tensors; workspace = the transformed filter (144 * Ci8 * Co4 bytes)
bool winograd5_applies(const Dims &d, int op);
size_t winograd5_ws_bytes(const Dims &d, int op);
hipError_t winograd5_fused(const Dims &d, int op, int b, const void *in, const void *w, void *out, float *ws,
                           bool filter_ready, hipStream_t s);
// BackwardFilter as F(5x5,2x2): workspace = the 36 K x C product planes (144 * K * C bytes); fp32 atomics
hipError_t winograd5_fused_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta, float *ws,
                                  hipStream_t s);

// zero-workspace implicit GEMM
hipError_t implicit_fwd(const Dims &d, int b, const void *x, const void *w, void *y, hipStream_t s);
hipError_t implicit_bwd_data(const Dims &d, int b, const void *dy, const void *w, void *dx, hipStream_t s);
// ws: only read in reproducible mode (implicit_det_ws_bytes(d, b) bytes)
hipError_t implicit_bwd_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                               float *ws, hipStream_t s);
size_t implicit_det_ws_bytes(const Dims &d, int b);
// BackwardData of a stride-1 layer as the Forward implicit GEMM of the mirrored layer (channels
// swapped, padding R-1-pad) on a copy of the filter with channels transposed and taps reversed; the
// copy (implicit_mirror_ws_bytes) sits at the head of the workspace and is kept when filter_ready
bool implicit_mirror_applies(const Dims &d, int op);
size_t implicit_mirror_ws_bytes(const Dims &d);
hipError_t implicit_bwd_data_mirror(const Dims &d, int b, const void *dy, const void *w, void *dx, void *ws,
                                    bool filter_ready, hipStream_t s);

// im2col into workspace + GEMM
size_t im2col_ws_bytes(const Dims &d, int b);
hipError_t im2col_fwd(const Dims &d, int b, const void *x, const void *w, void *y, float *ws, hipStream_t s);
hipError_t im2col_bwd_data(const Dims &d, int b, const void *dy, const void *w, void *dx, float *ws,
                           hipStream_t s);
hipError_t im2col_bwd_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                             float *ws, hipStream_t s);

// Winograd with tiles of mt = 2 or 4, 3x3 stride-1 layers: F(mt x mt, 3x3) for Forward and
// BackwardData, F(3x3, mt x mt) for BackwardFilter.  For the first two the transformed filter sits
// at the head of the workspace and depends on the layer and the operation only: filter_ready = true
// says that the previous launch on this workspace was the same operation on the same filter, so
// the filter transform is skipped.
bool winograd_applies(const Dims &d, int op);
size_t winograd_ws_bytes(const Dims &d, int op, int b, int mt);
hipError_t winograd_fwd(const Dims &d, int b, const void *x, const void *w, void *y, float *ws, bool filter_ready,
                        int mt, hipStream_t s);
hipError_t winograd_bwd_data(const Dims &d, int b, const void *dy, const void *w, void *dx, float *ws,
                             bool filter_ready, int mt, hipStream_t s);

hipError_t winograd_bwd_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                               float *ws, int mt, hipStream_t s);

// F(2x2,3x3) with the input and output transforms fused into the GEMM kernel: Forward (op 0) and
// BackwardData (op 1); the workspace holds the transformed filter only (independent of b).
bool winograd_fused_applies(const Dims &d, int op);
size_t winograd_fused_ws_bytes(const Dims &d, int op);
// BackwardFilter F(3x3,2x2) with both transforms fused: the workspace holds the 16 K x C product planes
size_t winograd_fused_filter_ws_bytes(const Dims &d);
hipError_t winograd_fused_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                                 float *ws, hipStream_t s);
hipError_t winograd_fused(const Dims &d, int op, int b, const void *in, const void *w, void *out, float *ws,
                          bool filter_ready, hipStream_t s);

// Tiled-FFT convolution (16x16 tiles), stride-1 layers with filters up to 9x9; filter_ready as
// for Winograd (Forward and BackwardData).
bool fft_applies(const Dims &d, int op);
size_t fft_ws_bytes(const Dims &d, int op, int b);
hipError_t fft_fwd(const Dims &d, int b, const void *x, const void *w, void *y, float *ws, bool filter_ready,
                   hipStream_t s);
hipError_t fft_bwd_data(const Dims &d, int b, const void *dy, const void *w, void *dx, float *ws, bool filter_ready,
                        hipStream_t s);
hipError_t fft_bwd_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta, float *ws,
                          hipStream_t s);

hipError_t fill_zero(float *p, size_t n, hipStream_t s);
// reduction splits of a BackwardFilter-shaped GEMM (small output, long reduction), `batch` of which
// run in one launch
int filter_splits(int M, int N, int Kd, int batch = 1);

// Dry-run support: while a log is installed (per host thread) every launcher appends a one-line
// description of the kernel it would launch and launches nothing.
struct LaunchLog {
    std::string text;
    int launches = 0;
    void add(const std::string &line)
    {
        if (!text.empty()) text += "; ";
        text += line;
        ++launches;
    }
};
LaunchLog *&launch_log();

// register-only MFMA loop (valu_per_mfma in {0, 2, 4, 8}); out holds blocks * 256 floats
hipError_t mfma_probe(int valu_per_mfma, int blocks, int iters, float *out, hipStream_t s);

}  // namespace ucd
