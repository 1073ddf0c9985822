// im2col into workspace + MFMA GEMM.  The workspace holds the column matrix
//   col[(c,r,s)][(n,p,q)] = x[n, c, p*sh - ph + r, q*sw - pw + s]   (0 outside the image)
// with leading dimension ld = b*P*Q rounded up to 4 floats, so its size grows with the
// micro-batch: 4 * C*R*S * ld bytes.
//   Forward        Y  = W[K x CRS] * col                     (epilogue scatters to NCHW)
//   BackwardData   col = W^T[CRS x K] * dY[K x bPQ], then dx = col2im(col) in gather form
//   BackwardFilter dW += dY[K x bPQ] * col^T                  (split over bPQ, fp32 atomics)
#include <type_traits>

#include "gemm_launch.hpp"
#include "kernels.h"

namespace ucd {

static inline int col_ld(const Dims &d, int b) { return (b * d.P * d.Q + 3) / 4 * 4; }

size_t im2col_ws_bytes(const Dims &d, int b) { return (size_t)4 * d.crs() * col_ld(d, b); }

struct ColParams {
    int C, H, W, R, S, sh, sw, ph, pw, P, Q;
    FastDiv pq, q, rs, s, hw, w;
    int n_cols, ld;
};

// one thread per column-matrix element, lanes along (n,p,q): coalesced writes, cached reads
template <class E>
__global__ __launch_bounds__(256) void im2col_kernel(const void *__restrict__ x, float *__restrict__ col,
                                                     ColParams p, int rows)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= p.ld) return;
    uint32_t n = 0, pix, op = 0, oq = 0;
    if (j < p.n_cols) {
        p.pq.divmod((uint32_t)j, n, pix);
        p.q.divmod(pix, op, oq);
    }
    for (int row = blockIdx.y; row < rows; row += gridDim.y) {
        float v = 0.f;
        if (j < p.n_cols) {
            uint32_t c, tap, r, s;
            p.rs.divmod((uint32_t)row, c, tap);
            p.s.divmod(tap, r, s);
            const int ih = (int)op * p.sh - p.ph + (int)r, iw = (int)oq * p.sw - p.pw + (int)s;
            if ((unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
                v = Elem<E>::get(x, (((size_t)n * p.C + c) * p.H + ih) * p.W + iw);
        }
        col[(size_t)row * p.ld + j] = v;
    }
}

// dx[n,c,h,w] = sum over the taps (r,s) that reach it of col[(c,r,s)][(n,p,q)]
template <class E>
__global__ __launch_bounds__(256) void col2im_kernel(const float *__restrict__ col, void *__restrict__ dx,
                                                     ColParams p, int total)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    uint32_t nc, pix, h, w, n, c;
    p.hw.divmod((uint32_t)i, nc, pix);
    p.w.divmod(pix, h, w);
    n = nc / (uint32_t)p.C;
    c = nc - n * (uint32_t)p.C;
    // only the taps of this pixel's stride phase can land: r = (h+ph) mod sh, then steps of sh
    float acc = 0.f;
    const int hp0 = (int)h + p.ph, wq0 = (int)w + p.pw;
    for (int r = hp0 % p.sh; r < p.R && r <= hp0; r += p.sh) {
        const int op = (hp0 - r) / p.sh;
        if (op >= p.P) continue;
        for (int s = wq0 % p.sw; s < p.S && s <= wq0; s += p.sw) {
            const int oq = (wq0 - s) / p.sw;
            if (oq >= p.Q) continue;
            acc += col[(size_t)((c * p.R + r) * p.S + s) * p.ld + (n * p.P + op) * p.Q + oq];
        }
    }
    Elem<E>::store(dx, i, acc);
}

static ColParams col_params(const Dims &d, int b)
{
    ColParams p;
    p.C = d.C; p.H = d.H; p.W = d.W; p.R = d.R; p.S = d.S; p.sh = d.sh; p.sw = d.sw; p.ph = d.ph; p.pw = d.pw;
    p.P = d.P; p.Q = d.Q;
    p.pq = FastDiv(d.P * d.Q); p.q = FastDiv(d.Q); p.rs = FastDiv(d.R * d.S); p.s = FastDiv(d.S);
    p.hw = FastDiv(d.H * d.W); p.w = FastDiv(d.W);
    p.n_cols = b * d.P * d.Q;
    p.ld = col_ld(d, b);
    return p;
}

template <class E>
static hipError_t run_im2col(const Dims &d, int b, const void *x, float *col, hipStream_t s)
{
    const ColParams p = col_params(d, b);
    dim3 grid((unsigned)((p.ld + 255) / 256), (unsigned)(d.crs() < 32768 ? d.crs() : 32768));
    if (LaunchLog *log = launch_log()) {
        log->add("im2col_kernel");
        return hipSuccess;
    }
    im2col_kernel<E><<<grid, 256, 0, s>>>(x, col, p, d.crs());
    return hipGetLastError();
}

template <class E>
static hipError_t im2col_fwd_t(const Dims &d, int b, const void *x, const void *w, void *y, float *ws, hipStream_t s)
{
    typedef Loaders<E> L;
    hipError_t e = run_im2col<E>(d, b, x, ws, s);
    if (e != hipSuccess) return e;
    GemmShape g{d.K, b * d.P * d.Q, d.crs()};
    KLaneParams pa{};
    pa.t = w; pa.bytes = wbytes(d); pa.row_stride = 1; pa.col_stride = d.crs();
    DenseParams pb{ws, (uint32_t)im2col_ws_bytes(d, b), col_ld(d, b)};
    EpiNCHWParams pe{};
    pe.out = y; pe.grid_hw = FastDiv(d.P * d.Q); pe.grid_w = FastDiv(d.Q);
    pe.M = d.K; pe.HWo = d.P * d.Q; pe.Wo = d.Q; pe.h0 = 0; pe.hs = 1; pe.w0 = 0; pe.ws = 1;
    return launch_gemm<L::template KLane0, DenseNLane, EpiNCHWT<E>, true>(pa, pb, pe, g, s);
}

hipError_t im2col_fwd(const Dims &d, int b, const void *x, const void *w, void *y, float *ws, hipStream_t s)
{
    return d.dtype == 1 ? im2col_fwd_t<bf16>(d, b, x, w, y, ws, s) : im2col_fwd_t<float>(d, b, x, w, y, ws, s);
}

template <class E>
static hipError_t im2col_bwd_data_t(const Dims &d, int b, const void *dy, const void *w, void *dx, float *ws,
                                    hipStream_t s)
{
    typedef Loaders<E> L;
    GemmShape g{d.crs(), b * d.P * d.Q, d.K};
    DenseParams pa{w, wbytes(d), d.crs()};
    GatherParams pb{};
    pb.t = dy; pb.bytes = ybytes(d, b); pb.Ct = d.K; pb.Ht = d.P; pb.Wt = d.Q;
    pb.grid_hw = FastDiv(d.P * d.Q); pb.grid_w = FastDiv(d.Q);
    pb.mul_h = 1; pb.add_h = 0; pb.mul_w = 1; pb.add_w = 0; pb.dir = 1;
    pb.taps = FastDiv(1); pb.taps_w = FastDiv(1);
    pb.n_tap_h = 1; pb.n_tap_w = 1; pb.shift_thread = 0; pb.shift_row = 0;
    EpiDenseParams pe{ws, col_ld(d, b)};
    hipError_t e;
    bool done = false;
    if constexpr (std::is_same<E, float>::value) {
        if (d.crs() % 4 == 0) {  // 16-byte loads of the fp32 filter matrix
            e = launch_gemm<DenseNLane, GatherNLane, EpiDense>(pa, pb, pe, g, s);
            done = true;
        }
    }
    if (!done) e = launch_gemm<L::template DenseNLaneS, L::template GatherNLane, EpiDense>(pa, pb, pe, g, s);
    if (e != hipSuccess) return e;
    const ColParams p = col_params(d, b);
    const int total = b * d.C * d.H * d.W;
    if (LaunchLog *log = launch_log()) {
        log->add("col2im_kernel");
        return hipSuccess;
    }
    col2im_kernel<E><<<(unsigned)((total + 255) / 256), 256, 0, s>>>(ws, dx, p, total);
    return hipGetLastError();
}

hipError_t im2col_bwd_data(const Dims &d, int b, const void *dy, const void *w, void *dx, float *ws,
                           hipStream_t s)
{
    return d.dtype == 1 ? im2col_bwd_data_t<bf16>(d, b, dy, w, dx, ws, s)
                        : im2col_bwd_data_t<float>(d, b, dy, w, dx, ws, s);
}

template <class E>
static hipError_t im2col_bwd_filter_t(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                                      float *ws, hipStream_t s)
{
    typedef Loaders<E> L;
    hipError_t e = run_im2col<E>(d, b, x, ws, s);
    if (e != hipSuccess) return e;
    if (beta == 0.f && (e = fill_zero(dw, (size_t)d.K * d.crs(), s)) != hipSuccess) return e;
    GemmShape g{d.K, d.crs(), b * d.P * d.Q};
    g.splits = filter_splits(g.M, g.N, g.Kd);
    KLaneParams pa{};
    pa.t = dy; pa.bytes = ybytes(d, b);
    pa.grid_hw = FastDiv(d.P * d.Q); pa.grid_w = FastDiv(d.Q);
    pa.col_taps = FastDiv(1); pa.col_taps_w = FastDiv(1);
    pa.n_stride = d.K * d.P * d.Q; pa.Ht = d.P; pa.Wt = d.Q;
    pa.mul_h = 1; pa.add_h = 0; pa.mul_w = 1; pa.add_w = 0;
    KLaneParams pb{};
    pb.t = ws; pb.bytes = (uint32_t)im2col_ws_bytes(d, b); pb.row_stride = 1; pb.col_stride = col_ld(d, b);
    EpiDenseParams pe{dw, d.crs()};
    return launch_gemm<L::template DyKLane, KLane0, EpiAtomic, true>(pa, pb, pe, g, s);
}

hipError_t im2col_bwd_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                             float *ws, hipStream_t s)
{
    return d.dtype == 1 ? im2col_bwd_filter_t<bf16>(d, b, x, dy, dw, beta, ws, s)
                        : im2col_bwd_filter_t<float>(d, b, x, dy, dw, beta, ws, s);
}

}  // namespace ucd
