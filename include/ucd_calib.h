/*
 * ucd -- calibration and introspection entry points.
 *
 * Not part of the method's boundary (that is ucd.h): these run or describe a single algorithm on a
 * single micro-batch, the unit the benchmark step of Section 3.2 times, and measure the matrix
 * ceiling the GEMM kernels are held against.  bench.py and the profiling runs use them; the
 * conventions (device pointers, caller-owned buffers, status codes, no synchronisation) are those
 * of ucd.h.
 */
#ifndef UCD_CALIB_H
#define UCD_CALIB_H

#include "ucd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Runs a single algorithm on one micro-batch of b samples starting at the given pointers
 * (already offset), bypassing plans: the unit the benchmark step times.  `a`, `bsrc`, `out`
 * are (x, w, y) for FWD, (dy, w, dx) for BWD_DATA, (x, dy, dw) for BWD_FILTER.  1 <= b <= layer->N
 * (UCD_E_INVALID otherwise): the buffers are taken to hold at least b samples. */
int ucd_run_micro(const ucd_layer_t *layer, int op, int algo, int b, const void *a,
                  const void *bsrc, void *out, float beta, void *ws, size_t ws_bytes,
                  void *stream);

/* Introspection: writes to buf (NUL-terminated, at most cap bytes) the kernels that
 * ucd_run_micro(layer, op, algo, b, ...) would launch, in order, separated by "; " (GEMM kernels
 * with their tile, loaders, epilogue, tile count, reduction splits and batch; BackwardFilter as
 * the accumulating beta = 1 call), and their number to *n_launches (may be NULL).  Launches
 * nothing.  Host only. */
int ucd_describe_micro(const ucd_layer_t *layer, int op, int algo, int b, char *buf, size_t cap,
                       int *n_launches);

/* Calibration of the roofline the GEMM kernels are held against (not part of the method):
 * enqueues a register-only loop of independent v_mfma_f32_32x32x2_f32 with `valu_per_mfma`
 * (0, 2, 4 or 8) ordinary vector FMAs interleaved per MFMA, on `blocks` workgroups of 256
 * threads, `iters` iterations of 16 MFMAs per wave.  100 + {0, 2, 4} runs the loop on 16 accumulator
 * tiles per wave (256 registers, so that only one wave fits a SIMD) instead of 4; 200 + {0, 2} does
 * the same with 4 consecutive MFMAs into each tile, every one depending on the one before (`iters`
 * must then be a multiple of 4; UCD_E_INVALID otherwise).  `scratch` is device memory of at least
 * blocks*1024 bytes (receives checksums).  *flops receives the MFMA flops one launch executes;
 * the caller times the launch. */
int ucd_mfma_probe(int valu_per_mfma, int blocks, int iters, void *scratch, size_t scratch_bytes,
                   void *stream, double *flops);

#ifdef __cplusplus
}
#endif
#endif /* UCD_CALIB_H */
