/*
 * ucd -- micro-batched convolution for MI355X (gfx950).
 *
 * C-ABI boundary of the library.  The method is the one of arXiv 1804.04806
 * ("mu-cuDNN"): a convolution layer's Forward, BackwardData and BackwardFilter
 * are executed as a sequence of micro-batches (Section 2), each micro-batch
 * running one of several equivalent algorithms with different workspace needs,
 * and a planner picks the division and the per-micro-batch algorithm that
 * minimise measured time under a workspace limit (Section 3).
 *
 * Conventions for every entry point
 *   - Tensors are dense, in DEVICE memory: X (N,C,H,W), filter W (K,C,R,S)
 *     with R the filter height and S its width, Y (N,K,P,Q) with
 *     P = floor((H + 2*pad_h - R)/stride_h) + 1 and Q likewise (Section 2 gives
 *     the NCHW / KCVU shapes; stride and zero padding are this library's
 *     reading, the operation is cross-correlation: no filter flip).
 *   - The caller owns every device buffer (tensors and workspace) and the
 *     stream.  The library allocates no device memory.  `stream` is a
 *     hipStream_t passed as void* (NULL = the default stream).
 *   - ucd_conv_* only enqueue work on `stream`; they never synchronise it.
 *     ucd_plan / ucd_plan_wd synchronise it to read event timings.
 *   - Return value: UCD_OK (0) or a negative ucd_status_t.  On failure no
 *     kernel has been launched by that call and *out arguments are untouched.
 *     Nothing throws or aborts across this boundary.
 *   - Host arrays (descriptors, tables, micro-configuration lists) are read
 *     during the call only.
 *   - Limits (checked on the host; UCD_E_INVALID / UCD_E_UNSUPPORTED, or
 *     UCD_WS_NA from ucd_workspace_size): filter extents R, S <= 31; every
 *     tensor slice one micro-batch touches (b*C*H*W, b*K*P*Q, K*C*R*S elements)
 *     and every workspace matrix below 2^29 - 2^16 elements, because the kernels
 *     address operands with 32-bit byte offsets; tensor pointers aligned to
 *     their element size, workspace pointers to 16 bytes (UCD_E_INVALID otherwise).
 */
#ifndef UCD_H
#define UCD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    UCD_OK = 0,
    UCD_E_INVALID = -1,      /* bad descriptor, enum value, size or micro-batch list */
    UCD_E_NULLPTR = -2,      /* a required pointer is NULL */
    UCD_E_UNSUPPORTED = -3,  /* algorithm does not apply to this layer / dtype not built */
    UCD_E_WS_TOO_SMALL = -4, /* workspace given is smaller than the plan needs */
    UCD_E_HIP = -5,          /* a HIP runtime call failed */
    UCD_E_NOMEM = -6,        /* host allocation failed */
    UCD_E_INFEASIBLE = -7    /* no configuration satisfies the limits */
} ucd_status_t;

/* dtype 0: every tensor fp32.
 * dtype 1: x, w, dy, y, dx hold bfloat16 (outputs rounded to nearest-even), dw is
 *          fp32 (it accumulates over micro-batches with beta = 1) and so is every workspace
 *          matrix.  Products of bf16 values are exact in fp32 and all accumulation is fp32
 *          (on the bf16 matrix instructions where both operands of a GEMM are bf16 tensors),
 *          so results differ from dtype 0 on the same values only by summation order and by
 *          the rounding of y / dx.
 * Layout NCHW / KCRS, dense, groups = 1, dilation = 1. */
typedef struct {
    int32_t N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, dtype;
} ucd_layer_t;

/* The three operations of Section 2. */
enum { UCD_FWD = 0, UCD_BWD_DATA = 1, UCD_BWD_FILTER = 2, UCD_N_OP = 3 };

/* Equivalent algorithms, differing in workspace need (the role cuDNN's algorithm list plays
 * in Section 1): implicit GEMM (no workspace), im2col into workspace + GEMM, Winograd F(2x2,3x3)
 * and Winograd F(4x4,3x3) with transform buffers in workspace (3x3 stride-1 layers only, all
 * three operations, BackwardFilter as F(3x3,2x2) / F(3x3,4x4); the larger tile does 36 products
 * per 16 outputs instead of 16 per 4 and needs less workspace per sample, at a looser rounding
 * error). */
enum {
    UCD_ALGO_IMPLICIT = 0, UCD_ALGO_IM2COL = 1, UCD_ALGO_WINOGRAD = 2, UCD_ALGO_WINOGRAD4 = 3,
    UCD_ALGO_FFT = 4,  /* tiled FFT (16x16 tiles): stride-1 layers, filters up to 9x9, all three
                        * operations; the largest workspace of all (144 frequency planes) */
    UCD_ALGO_WINOGRAD_FUSED = 5,  /* Winograd F(2x2,3x3) (BackwardFilter: F(3x3,2x2)) with the data
                        * transforms inside the GEMM kernel: the workspace holds the transformed filter
                        * (BackwardFilter: the 16 K x C product planes) only, whatever the micro-batch size.
                        * 3x3 stride-1 layers; also BackwardData of strided layers whose output phases
                        * each see three filter taps per axis (11x11 stride 4, 5x5 stride 2, 7x7 stride 3):
                        * all phases together are one 3x3 stride-1 convolution over dy */
    UCD_ALGO_IMPLICIT_MIRROR = 6, /* BackwardData of stride-1 layers (padding <= filter extent - 1) as the
                                     Forward implicit GEMM of the mirrored layer on a copy of the
                                     filter with channels transposed and taps reversed: workspace =
                                     that copy, whatever the micro-batch size */
    UCD_ALGO_WINOGRAD5_FUSED = 7, /* Winograd F(2x2,5x5) (BackwardFilter: F(5x5,2x2)) with the data transforms
                                     inside the GEMM kernel: 5x5 stride-1 layers with horizontal padding 2,
                                     fp32 tensors; workspace = the transformed filter (BackwardFilter: the
                                     36 K x C product planes) */
    UCD_N_ALGO = 8
};

/* Batch-size policies of Section 3.4: which micro-batch sizes get benchmarked: only B; the powers
 * of two below B and B itself; every size 1..B. */
enum { UCD_POLICY_UNDIVIDED = 0, UCD_POLICY_POW2 = 1, UCD_POLICY_ALL = 2 };

/* A micro-configuration (Section 3.1): algorithm and micro-batch size. */
typedef struct { int32_t algo, batch; } ucd_micro_t;

/* A configuration: ordered list of micro-configurations, plus the layer and operation it is
 * for.  Opaque, host memory owned by the library, freed by ucd_plan_destroy. */
typedef struct ucd_plan ucd_plan_t;

#define UCD_TIME_INF UINT64_MAX  /* "not benchmarked / does not apply" in timing tables */
#define UCD_WS_NA SIZE_MAX       /* "algorithm does not apply" in workspace tables */

const char *ucd_strerror(int status);
int ucd_version(void);

/* Run-to-run reproducibility.  By default some launches sum partial results with hardware fp32
 * atomics, whose order of arrival differs from run to run, so these outputs are reproducible only
 * up to rounding (and micro-batched == undivided likewise):
 *   - BackwardFilter, every algorithm: the reduction over b*P*Q is split over workgroups whenever
 *     it is long enough (always at the benchmark sizes), and micro-batches accumulate into dw;
 *   - Forward / BackwardData, implicit GEMM (also on the mirrored filter copy), fp32 tensors only: when the output has fewer than 768
 *     tiles the reduction over C*R*S is split the same way into a zero-filled output, and when the
 *     tile count is not a multiple of 256 the last tiles' reductions are spread over several
 *     workgroups.
 * Everything else (im2col, Winograd and FFT Forward / BackwardData; implicit-GEMM Forward /
 * BackwardData with bf16 tensors or without the splits above) adds each output once and is bit
 * reproducible.
 * ucd_set_deterministic(1) switches the library (process-wide) to reproducible execution: Forward /
 * BackwardData never split a reduction, and BackwardFilter is offered by the implicit GEMM alone,
 * which then writes each reduction chunk's partial result to workspace and sums the chunks in a
 * fixed order (ucd_workspace_size reports those bytes, at most 32 MiB, so the planners price
 * them; the other algorithms report UCD_WS_NA for BackwardFilter).  Results are then bit-identical
 * from run to run for a given configuration.  Timings of the two modes are cached apart.  Plans
 * made in one mode must be executed in that mode (a plan's workspace need differs).
 * on < 0 only queries.  Returns the previous setting. */
int ucd_set_deterministic(int on);

/* Bytes of workspace algorithm `algo` needs for operation `op` at micro-batch size b (the
 * quantity compared with the limit M in step 1 of the WR algorithm, Section 3.2):
 *   implicit   0 (reproducible mode, BackwardFilter: 4*K*C*R*S bytes per reduction chunk, see
 *              ucd_set_deterministic)
 *   implicit GEMM on a mirrored filter copy (BackwardData only)   e * K*C*R*S rounded up to 16,
 *              e = 4 (fp32 tensors) or 2 (bf16)
 *   im2col     4 * C*R*S * ld,  ld = b*P*Q rounded up to 4
 *   Winograd   4 * a*a * (Ci*Co4 + ld*(C + K)) with a = 4 (F(2x2,3x3)) or 6 (F(4x4,3x3)),
 *              ld = b * ceil(Ho/m) * ceil(Wo/m) rounded up to 4 (m = a - 2), where (Ci, Co, Ho, Wo)
 *              = (C, K, P, Q) for Forward and (K, C, H, W) for BackwardData, Co4 = Co rounded up
 *              to 4; BackwardFilter: K*C in place of Ci*Co4, tiles over (P, Q)
 *   Winograd, fused transforms   64 * Ci8*Co4 (the transformed filter, Ci8 = Ci rounded up to 8);
 *              BackwardFilter 64 * K*C; BackwardData of a strided layer with three filter taps per
 *              output phase and axis (ceil(R/stride_h) = ceil(S/stride_w) = 3): Ci = K and
 *              Co = C*stride_h*stride_w
 *   Winograd F(2x2,5x5), fused transforms   144 * Ci8*Co4; BackwardFilter 144 * K*C
 *   FFT        4 * 144 * (2Ci*M4 + ld*(2Ci + 2Co)), M4 = 2Co rounded up to 4, ld = b *
 *              ceil(Ho/(17-R)) * ceil(Wo/(17-S)) rounded up to 4, (Ci, Co, Ho, Wo) as for Winograd;
 *              BackwardFilter: 4*K*C in place of 2Ci*M4, tiles over (P, Q)
 * Returns UCD_WS_NA if the algorithm does not apply or an argument is invalid.  Host only. */
size_t ucd_workspace_size(const ucd_layer_t *layer, int op, int algo, int b);

/* ---- planners on a given timing table (pure host, no GPU needed) ------------------------- */

/* WR planner (Section 3.2, steps 2-3): T(b) = min over b_mu of T_mu(b_mu) + T(b - b_mu), T(0)=0,
 * where T_mu(b) is the least t_ns[a][b] over algorithms a with ws[a][b] <= ws_limit, restricted
 * to the micro-batch sizes the policy allows.
 *   t_ns, ws : row-major [n_algo][B+1], column 0 unused; UCD_TIME_INF / UCD_WS_NA mark holes.
 * On success *out is a plan with no layer attached (query only, cannot be executed).
 * Ties: the largest first micro-batch, then the lowest algorithm id.  UCD_E_INFEASIBLE if no
 * division of B is feasible. */
int ucd_plan_from_table(int B, size_t ws_limit, int policy, int n_algo,
                        const uint64_t *t_ns, const size_t *ws, ucd_plan_t **out);

/* Desirable configuration set C(B) of Section 3.3: the set-valued variant of the WR programme,
 * pruned at every b to the Pareto front in (time, workspace), where a configuration's time is
 * the sum and its workspace the maximum over its micro-configurations.  Writes up to `cap`
 * points, sorted by increasing workspace (hence decreasing time), to front_t / front_ws and
 * the number found to *n (which may exceed cap: call again with a bigger cap). */
int ucd_desirable_from_table(int B, size_t ws_limit, int policy, int n_algo,
                             const uint64_t *t_ns, const size_t *ws,
                             uint64_t *front_t, size_t *front_ws, int cap, int *n);

/* WD 0-1 programme (Section 3.3, Eq. 1-4) over given desirable sets: choose one point per
 * kernel, sum of workspaces <= budget, least sum of times.  Points of kernel k are
 * front_t/front_ws[offset_k .. offset_k + front_n[k]), offsets being the running sum of front_n.
 * Exact.  choice[k] receives the chosen index within kernel k, *total_t the optimum. */
int ucd_wd_solve(int n_kernels, const int *front_n, const uint64_t *front_t,
                 const size_t *front_ws, size_t budget, int *choice, uint64_t *total_t);

/* WD planner on given tables: kernel k has mini-batch B[k] and tables at t_ns/ws + tab_off[k]
 * (each [n_algo][B[k]+1]).  Builds every desirable set, solves the programme, and returns one
 * layer-less plan per kernel in plans[k] and its segment offset (bytes, 256-aligned running
 * sum in kernel order) in ws_offsets[k].  Segment sizes are rounded up to 256 bytes before
 * they are summed against total_ws. */
int ucd_plan_wd_from_tables(int n_kernels, const int *B, int n_algo, const size_t *tab_off,
                            const uint64_t *t_ns, const size_t *ws, size_t total_ws, int policy,
                            ucd_plan_t **plans, size_t *ws_offsets);

/* ---- plans ------------------------------------------------------------------------------ */

/* A forced configuration (for tests and for undivided baselines): micro[0..n) must have positive
 * sizes summing to layer->N and algorithms that apply to (layer, op). */
int ucd_plan_fixed(const ucd_layer_t *layer, int op, const ucd_micro_t *micro, int n,
                   ucd_plan_t **out);

/* Reads a plan: copies up to cap micro-configurations to `micro` (may be NULL if cap == 0),
 * their count to *n, the planner's predicted cost (sum of table times; 0 for fixed plans) to
 * *cost_ns and the workspace the plan needs (largest over its parts) to *ws_bytes.
 * Any out pointer may be NULL. */
int ucd_plan_query(const ucd_plan_t *plan, ucd_micro_t *micro, int cap, int *n,
                   uint64_t *cost_ns, size_t *ws_bytes);

void ucd_plan_destroy(ucd_plan_t *plan);

/* ---- on-device benchmark + WR plan (Section 3.2, steps 1-3) --------------------------------
 * Times every algorithm that applies and fits ws_limit at every micro-batch size the policy
 * allows, on the caller's buffers, keeps the timings in a process-wide cache keyed by
 * (layer shape without N, op, algo, b) so that identical layers are timed once (Section 3.4),
 * then runs the WR programme on that table.
 *   x  : device, N*C*H*W floats      y : device, N*K*P*Q floats      w : device, K*C*R*S floats
 *   ws : device, at least ws_limit bytes (may be NULL when ws_limit == 0)
 * The operation's output buffer is clobbered (FWD: y, BWD_DATA: x, BWD_FILTER: w); the other
 * two are only read.  For BWD_FILTER `w` stands in for dw and must hold K*C*R*S fp32 values
 * whatever the dtype.  Each timing is, after one warm-up run, the time per run of 2-8 runs
 * launched back to back on consecutive micro-batches of the buffers, in integer ns.  The
 * planned configuration's micro-batches are stored grouped by algorithm and run in that order
 * (consecutive Winograd micro-batches transform the filter once, so a configuration can run
 * slightly faster than the sum of its standalone timings). */
int ucd_plan(const ucd_layer_t *layer, int op, size_t ws_limit, int policy,
             void *x, void *w, void *y, void *ws, void *stream, ucd_plan_t **out);

/* WD planner on the device (Section 3.3): benchmarks like ucd_plan (limit = total_ws) for each
 * of the n_kernels (layers[k], ops[k]) kernels, using the same scratch tensors for all of them
 * (each must be large enough for the largest layer; capacities in bytes are checked; the w
 * scratch is sized as K*C*R*S fp32 values for every dtype, since BackwardFilter writes dw there), then
 * builds desirable sets and solves the 0-1 programme.  plans[k] are executable; kernel k must
 * be run with workspace pointer ws_base + ws_offsets[k]. */
int ucd_plan_wd(const ucd_layer_t *layers, const int *ops, int n_kernels, size_t total_ws,
                int policy, void *x, size_t x_cap, void *w, size_t w_cap, void *y, size_t y_cap,
                void *ws, void *stream, ucd_plan_t **plans, size_t *ws_offsets);

/* Copies the cached timings of (layer, op) into t_ns[algo*(cap_b+1) + b] and the workspace
 * formula into ws[...] for b = 1..cap_b; entries never timed are UCD_TIME_INF.  Host only. */
int ucd_bench_table(const ucd_layer_t *layer, int op, uint64_t *t_ns, size_t *ws, int cap_b);

/* Forgets every cached timing. */
void ucd_bench_clear(void);

/* File-backed benchmark database (Section 3.4: timings are kept in a file so that benchmarking
 * can happen offline and be shared between identical GPUs).
 * ucd_bench_save writes every cached timing to a text file; ucd_bench_load merges a file into
 * the cache (*n_loaded, may be NULL, receives the number of timings read) and refuses, with
 * UCD_E_UNSUPPORTED, a file taken on a different device than the current one (a process without
 * a GPU accepts any file).  ucd_bench_put injects one timing by hand.  Host only. */
int ucd_bench_save(const char *path);
int ucd_bench_load(const char *path, int *n_loaded);
int ucd_bench_put(const ucd_layer_t *layer, int op, int algo, int b, uint64_t t_ns);

/* WR plan from the cache alone (offline planning, no GPU work): like ucd_plan, but (algorithm, b)
 * pairs without a cached timing count as not benchmarked.  The plan is executable. */
int ucd_plan_cached(const ucd_layer_t *layer, int op, size_t ws_limit, int policy, ucd_plan_t **out);

/* ---- execution (Section 2: micro-batches run one after another on one stream, sharing one
 * workspace; sample n of a micro-batch starting at offset o is sample o+n of the tensors) --- */

/* y = conv(x, w).  Overwrites y. */
int ucd_conv_fwd(const ucd_plan_t *plan, const void *x, const void *w, void *y,
                 void *ws, size_t ws_bytes, void *stream);

/* ucd_conv_fwd for callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the workspace is an
 * array of UCD_STATIC_WS_BYTES that the library's code object holds on every GPU it is loaded on,
 * from load to process end.  Allocates nothing (no hipMalloc / hipFree, no allocating library
 * call); the array's address on the current device is looked up on the first call on that device.
 * A plan that needs more than UCD_STATIC_WS_BYTES is refused with UCD_E_WS_TOO_SMALL before any
 * launch.  Every call on one GPU uses the same array, which keeps the previous call's contents
 * (every algorithm writes all it reads, nothing needs clearing): calls that overlap on one GPU
 * (different streams, or threads) race; calls on one stream are ordered and safe. */
#define UCD_STATIC_WS_BYTES ((size_t)64 << 20)
int ucd_conv_fwd_static_ws(const ucd_plan_t *plan, const void *x, const void *w, void *y, void *stream);

/* dx = adjoint of Forward with respect to x, applied to dy.  Overwrites all of dx (input pixels
 * no filter tap reaches become 0). */
int ucd_conv_bwd_data(const ucd_plan_t *plan, const void *dy, const void *w, void *dx,
                      void *ws, size_t ws_bytes, void *stream);

/* dw = beta * dw + sum over samples, beta in {0, 1}; beta = 0 ignores dw's old contents.
 * The first micro-batch uses the caller's beta, later ones accumulate with output scale 1. */
int ucd_conv_bwd_filter(const ucd_plan_t *plan, const void *x, const void *dy, void *dw,
                        float beta, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* UCD_H */
