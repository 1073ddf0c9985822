// Tiled-FFT convolution for stride-1 layers, Forward and BackwardData: the workspace-hungry
// algorithm whose feasibility micro-batching changes most (Section 4 of the paper: FFT tiling fits
// the limit only at small micro-batches).  16x16 tiles of the input, each producing a
// (17-R) x (17-S) tile of the output:
//   out_tile = IDFT( DFT(in_tile) . conj(DFT(filter zero-padded to 16x16)) )   summed over channels
// A real tile's transform is Hermitian, so 16 x 9 = 144 frequencies are kept.  Per frequency f the
// channel sum is a complex matrix product  Z_f[co][j] = sum_ci conj(U_f[co][ci]) V_f[ci][j]  over
// the tiles j of the micro-batch, run as one real GEMM on stacked real and imaginary parts:
//   [Zr; Zi] = [[Ur, Ui], [-Ui, Ur]] [Vr; Vi]
// Everything lives in the caller's workspace:
//   AT[144][2Ci][M4]   the 2Co x 2Ci block matrix above, stored reduction-major (M4 = 2Co up to 4)
//   B [144][2Ci][ld]   input transforms, ld = b*T rounded up to 4, T = tiles per image
//   Z [144][2Co][ld]   the products
// The transforms are separable 16-point FFTs in registers (fft16.hpp) with one pass through LDS.
// BackwardData is the same pipeline on dy with the filter's two channel indices swapped and its
// taps reversed, and padding (R-1-pad_h, S-1-pad_w).
//
// BackwardFilter: a tile's filter gradient is the correlation of its 16x16 tile of x with its
// (17-R) x (17-S) tile of dy (zero-padded to 16x16), so in the frequency domain
//   Mw_f[k][c] = sum over tiles j of V_f[c][j] conj(D_f[k][j]),    dw = beta*dw + IDFT(Mw)[0..R)[0..S)
// with V and D the input transforms of x and dy.  One real GEMM per frequency, reduction over the
// tiles (split, atomics), gives the four real products  P = [Dr; Di] [Vr; Vi]^T  (2K x 2C), which
// the output kernel combines (Mr = Prr + Pii, Mi = Pri - Pir) before it inverts:
//   Mw[144][2K][2C]    V[144][2C][ld]    D[144][2K][ld]
#include "fft16.hpp"
#include "gemm_launch.hpp"
#include "kernels.h"

namespace ucd {

constexpr int kFftN = 16, kFftHalf = 9, kFftFreqs = kFftN * kFftHalf;
constexpr int kFftTilesPerBlock = 32;  // tiles (filters, channel pairs) per workgroup: 128-byte rows of lanes
constexpr int kFftThreads = kFftTilesPerBlock * kFftN;  // one thread per (tile, row)

struct FftGeom {
    int Ci, Co, Hi, Wi, Ho, Wo, pad_h, pad_w, R, S;
    int Th, Tw, TH, TW, T;  // output tile, tiles per image
    int M4, ld;
    int win_h, win_w;  // rows / columns of a tile that are read (the rest of the 16x16 tile is zero)
    bool transposed;   // BackwardData: filter read as w[ci][co] with reversed taps
};

static FftGeom fft_geom(const Dims &d, int op, int b)
{
    FftGeom g;
    if (op == 0) {
        g.Ci = d.C; g.Co = d.K; g.Hi = d.H; g.Wi = d.W; g.Ho = d.P; g.Wo = d.Q;
        g.pad_h = d.ph; g.pad_w = d.pw; g.transposed = false;
    } else {
        g.Ci = d.K; g.Co = d.C; g.Hi = d.P; g.Wi = d.Q; g.Ho = d.H; g.Wo = d.W;
        g.pad_h = d.R - 1 - d.ph; g.pad_w = d.S - 1 - d.pw; g.transposed = true;
    }
    g.R = d.R; g.S = d.S;
    g.Th = kFftN + 1 - d.R; g.Tw = kFftN + 1 - d.S;
    g.TH = (g.Ho + g.Th - 1) / g.Th; g.TW = (g.Wo + g.Tw - 1) / g.Tw; g.T = g.TH * g.TW;
    g.M4 = (2 * g.Co + 3) / 4 * 4;
    g.ld = (b * g.T + 3) / 4 * 4;
    g.win_h = g.win_w = kFftN;
    return g;
}

bool fft_applies(const Dims &d, int op)
{
    if (op < 0 || op > 2) return false;
    if (d.sh != 1 || d.sw != 1) return false;
    if (d.R > 9 || d.S > 9 || d.R * d.S < 2) return false;  // output tiles of at least 8 x 8
    return d.ph <= d.R - 1 && d.pw <= d.S - 1;
}

size_t fft_ws_bytes(const Dims &d, int op, int b)
{
    if (op == 2) {  // Mw, V, D
        const FftGeom g = fft_geom(d, 0, b);
        return (size_t)4 * kFftFreqs * ((size_t)4 * d.K * d.C + (size_t)g.ld * (2 * d.C + 2 * d.K));
    }
    const FftGeom g = fft_geom(d, op, b);
    return (size_t)4 * kFftFreqs * ((size_t)2 * g.Ci * g.M4 + (size_t)g.ld * (2 * g.Ci + 2 * g.Co));
}

// AT[f][kk][m] for all 144 frequencies: U = the 2-D transform of the filter zero-padded to 16x16.
// A workgroup transforms the filters of 32 consecutive output channels for one input channel:
// thread (filter, row) does the row FFT of the padded filter, the results cross through LDS,
// thread (frequency column, filter) does the column FFT and writes the four entries of the block
// matrix with lanes along the output channel.
template <class E>
__global__ __launch_bounds__(kFftThreads) void fft_filter_kernel(const void *__restrict__ w, float *__restrict__ AT,
                                                         FftGeom g)
{
    __shared__ float sre[kFftTilesPerBlock * kFftHalf * kFftN], sim[kFftTilesPerBlock * kFftHalf * kFftN];
    const int tid = threadIdx.x;
    const int ci = blockIdx.y;
    const int co0 = blockIdx.x * kFftTilesPerBlock;
    {
        const int fa = tid / kFftN, ia = tid % kFftN;  // filter in the block, row of the padded filter
        const int co = co0 + fa;
        const bool row_ok = co < g.Co && ia < g.R;
        const int taps = g.R * g.S;
        // row ia of g[co][ci]: w[co][ci][ia][.] for Forward, w[ci][co][R-1-ia][S-1-.] for BackwardData
        const size_t base = g.transposed ? (size_t)(ci * g.Co + (row_ok ? co : 0)) * taps + (row_ok ? g.R - 1 - ia : 0) * g.S
                                         : (size_t)((row_ok ? co : 0) * g.Ci + ci) * taps + (row_ok ? ia : 0) * g.S;
        float re[kFftN], im[kFftN];
#pragma unroll
        for (int c = 0; c < kFftN; ++c) {
            re[c] = (row_ok && c < g.S) ? Elem<E>::get(w, base + (g.transposed ? g.S - 1 - c : c)) : 0.f;
            im[c] = 0.f;
        }
        fft16<-1>(re, im);
#pragma unroll
        for (int v = 0; v < kFftHalf; ++v) {
            sre[(fa * kFftHalf + v) * kFftN + ia] = re[v];
            sim[(fa * kFftHalf + v) * kFftN + ia] = im[v];
        }
    }
    __syncthreads();
    const int vb = tid / kFftTilesPerBlock, fb = tid % kFftTilesPerBlock;
    const int co = co0 + fb;
    if (vb < kFftHalf && co < g.Co) {
        float re[kFftN], im[kFftN];
#pragma unroll
        for (int r = 0; r < kFftN; ++r) {
            re[r] = sre[(fb * kFftHalf + vb) * kFftN + r];
            im[r] = sim[(fb * kFftHalf + vb) * kFftN + r];
        }
        fft16<-1>(re, im);
        const size_t plane = (size_t)2 * g.Ci * g.M4;
#pragma unroll
        for (int u = 0; u < kFftN; ++u) {
            float *dst = AT + (size_t)(u * kFftHalf + vb) * plane;
            dst[(size_t)ci * g.M4 + co] = re[u];
            dst[(size_t)(g.Ci + ci) * g.M4 + co] = im[u];
            dst[(size_t)ci * g.M4 + g.Co + co] = -im[u];
            dst[(size_t)(g.Ci + ci) * g.M4 + g.Co + co] = re[u];
        }
    }
}

// B[f][ci][j] (real part) and B[f][Ci + ci][j] (imaginary part) of the 16x16 input tile j.  A
// workgroup transforms 32 tiles of one channel: thread (tile, row) does the row FFT, the results
// cross through LDS, thread (frequency column, tile) does the column FFT and writes with lanes
// along the tile index.
template <class E>
__global__ __launch_bounds__(kFftThreads) void fft_input_kernel(const void *__restrict__ x, float *__restrict__ B, FftGeom g,
                                                        FastDiv divT, FastDiv divTW, int n_tiles)
{
    __shared__ float sre[kFftTilesPerBlock * kFftHalf * kFftN], sim[kFftTilesPerBlock * kFftHalf * kFftN];
    const int tid = threadIdx.x;
    const int j0 = blockIdx.x * kFftTilesPerBlock;
    // row phase: tile ta, row ia
    const int ta = tid / kFftN, ia = tid % kFftN;
    const int ja = j0 + ta;
    uint32_t n = 0, t, th = 0, tw = 0;
    const bool live = ja < n_tiles;
    if (live) {
        divT.divmod((uint32_t)ja, n, t);
        divTW.divmod(t, th, tw);
    }
    const int h = (int)th * g.Th - g.pad_h + ia, w0 = (int)tw * g.Tw - g.pad_w;
    const bool row_ok = live && (unsigned)h < (unsigned)g.Hi && ia < g.win_h;
    // column phase: frequency column vb, tile tb (threads 0..143)
    const int vb = tid / kFftTilesPerBlock, tb = tid % kFftTilesPerBlock;
    const int jb = j0 + tb;
    const size_t plane = (size_t)2 * g.Ci * g.ld;
    for (int ci = blockIdx.y; ci < g.Ci; ci += gridDim.y) {
        float re[kFftN], im[kFftN];
        const size_t src = (((size_t)n * g.Ci + ci) * g.Hi + (row_ok ? h : 0)) * g.Wi;
#pragma unroll
        for (int c = 0; c < kFftN; ++c) {
            const int ww = w0 + c;
            re[c] = (row_ok && c < g.win_w && (unsigned)ww < (unsigned)g.Wi) ? Elem<E>::get(x, src + ww) : 0.f;
            im[c] = 0.f;
        }
        fft16<-1>(re, im);
#pragma unroll
        for (int v = 0; v < kFftHalf; ++v) {
            sre[(ta * kFftHalf + v) * kFftN + ia] = re[v];
            sim[(ta * kFftHalf + v) * kFftN + ia] = im[v];
        }
        __syncthreads();
        if (vb < kFftHalf && jb < g.ld) {
#pragma unroll
            for (int r = 0; r < kFftN; ++r) {
                re[r] = sre[(tb * kFftHalf + vb) * kFftN + r];
                im[r] = sim[(tb * kFftHalf + vb) * kFftN + r];
            }
            fft16<-1>(re, im);
            float *dst = B + (size_t)ci * g.ld + jb;
#pragma unroll
            for (int u = 0; u < kFftN; ++u) {
                float *p = dst + (size_t)(u * kFftHalf + vb) * plane;
                p[0] = re[u];
                p[(size_t)g.Ci * g.ld] = im[u];
            }
        }
        __syncthreads();
    }
}

// out tile = the real inverse transform of Z[., co, j] (rows co and Co + co hold the real and the
// imaginary part).  Thread (frequency column, tile) inverts along u, the results cross through
// LDS, thread (tile, row a) completes the Hermitian half along v, inverts and stores its row.
template <class E>
__global__ __launch_bounds__(kFftThreads) void fft_output_kernel(const float *__restrict__ Z, void *__restrict__ out,
                                                         FftGeom g, FastDiv divT, FastDiv divTW, int n_tiles)
{
    __shared__ float sre[kFftTilesPerBlock * kFftN * kFftHalf], sim[kFftTilesPerBlock * kFftN * kFftHalf];
    const int tid = threadIdx.x;
    const int j0 = blockIdx.x * kFftTilesPerBlock;
    const int va = tid / kFftTilesPerBlock, ta = tid % kFftTilesPerBlock;
    const int ja = j0 + ta;
    const int tb = tid / kFftN, ab = tid % kFftN;
    const int jb = j0 + tb;
    uint32_t n = 0, t, th = 0, tw = 0;
    const bool live = jb < n_tiles;
    if (live) {
        divT.divmod((uint32_t)jb, n, t);
        divTW.divmod(t, th, tw);
    }
    const int ho = (int)th * g.Th + ab, wo0 = (int)tw * g.Tw;
    const bool row_ok = live && ab < g.Th && ho < g.Ho;
    const size_t plane = (size_t)2 * g.Co * g.ld;
    for (int co = blockIdx.y; co < g.Co; co += gridDim.y) {
        float re[kFftN], im[kFftN];
        if (va < kFftHalf) {
            const bool ok = ja < n_tiles;
            const float *src = Z + (size_t)co * g.ld + (ok ? ja : 0);
#pragma unroll
            for (int u = 0; u < kFftN; ++u) {
                const float *p = src + (size_t)(u * kFftHalf + va) * plane;
                re[u] = ok ? p[0] : 0.f;
                im[u] = ok ? p[(size_t)g.Co * g.ld] : 0.f;
            }
            fft16<1>(re, im);
#pragma unroll
            for (int a = 0; a < kFftN; ++a) {
                sre[(ta * kFftN + a) * kFftHalf + va] = re[a];
                sim[(ta * kFftN + a) * kFftHalf + va] = im[a];
            }
        }
        __syncthreads();
#pragma unroll
        for (int v = 0; v < kFftHalf; ++v) {
            re[v] = sre[(tb * kFftN + ab) * kFftHalf + v];
            im[v] = sim[(tb * kFftN + ab) * kFftHalf + v];
        }
#pragma unroll
        for (int v = kFftHalf; v < kFftN; ++v) {  // P[a][16 - v] = conj(P[a][v])
            re[v] = re[kFftN - v];
            im[v] = -im[kFftN - v];
        }
        fft16<1>(re, im);
        if (row_ok) {
            const size_t dst = (((size_t)n * g.Co + co) * g.Ho + ho) * g.Wo + wo0;
#pragma unroll
            for (int c = 0; c < kFftN; ++c)
                if (c < g.Tw && wo0 + c < g.Wo) Elem<E>::store(out, dst + c, re[c] * (1.f / 256.f));
        }
        __syncthreads();
    }
}

template <class E>
static hipError_t fft_run(const Dims &d, int op, int b, const void *in, const void *w, void *out, float *ws,
                          bool filter_ready, hipStream_t s)
{
    const FftGeom g = fft_geom(d, op, b);
    const int n_tiles = b * g.T;
    float *AT = ws;
    float *B = AT + (size_t)kFftFreqs * 2 * g.Ci * g.M4;
    float *Z = B + (size_t)kFftFreqs * 2 * g.Ci * g.ld;
    const FastDiv divT(g.T), divTW(g.TW);

    LaunchLog *log = launch_log();
    hipError_t e = hipSuccess;
    if (filter_ready) {
        // the transformed filter is still at the head of the workspace from the previous micro-batch
    } else if (log) {
        log->add("fft_filter_kernel");
    } else {
        const dim3 gf((unsigned)((g.Co + kFftTilesPerBlock - 1) / kFftTilesPerBlock), (unsigned)g.Ci);
        fft_filter_kernel<E><<<gf, kFftThreads, 0, s>>>(w, AT, g);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)((g.ld + kFftTilesPerBlock - 1) / kFftTilesPerBlock);
    if (log) {
        log->add("fft_input_kernel");
    } else {
        fft_input_kernel<E><<<dim3(blocks, (unsigned)(g.Ci < 1024 ? g.Ci : 1024)), kFftThreads, 0, s>>>(in, B, g, divT, divTW,
                                                                                              n_tiles);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    GemmShape gs{2 * g.Co, n_tiles, 2 * g.Ci};
    gs.batch = kFftFreqs;
    gs.a_batch = (long)2 * g.Ci * g.M4;
    gs.b_batch = (long)2 * g.Ci * g.ld;
    gs.c_batch = (long)2 * g.Co * g.ld;
    DenseParams pa{AT, (uint32_t)(gs.a_batch * 4), g.M4};
    DenseParams pb{B, (uint32_t)(gs.b_batch * 4), g.ld};
    EpiDenseParams pe{Z, g.ld};
    if ((e = launch_gemm<DenseNLane, DenseNLane, EpiDense>(pa, pb, pe, gs, s)) != hipSuccess) return e;
    if (log) {
        log->add("fft_output_kernel");
        return hipSuccess;
    }
    const unsigned oblocks = (unsigned)((n_tiles + kFftTilesPerBlock - 1) / kFftTilesPerBlock);
    fft_output_kernel<E><<<dim3(oblocks, (unsigned)(g.Co < 1024 ? g.Co : 1024)), kFftThreads, 0, s>>>(Z, out, g, divT, divTW,
                                                                                            n_tiles);
    return hipGetLastError();
}

// dw[k][c] = beta * dw[k][c] + the first R x S values of the inverse transform of
// Mw[.][k][c] = (Prr + Pii) + i (Pri - Pir), P = the 2K x 2C product matrix of one frequency.
// A workgroup handles 32 consecutive input channels of one output channel.
__global__ __launch_bounds__(kFftThreads) void fft_dw_kernel(const float *__restrict__ P, float *__restrict__ dw, int K, int C,
                                                     int R, int S, float beta)
{
    __shared__ float sre[kFftTilesPerBlock * kFftN * kFftHalf], sim[kFftTilesPerBlock * kFftN * kFftHalf];
    const int tid = threadIdx.x;
    const int k = blockIdx.y, c0 = blockIdx.x * kFftTilesPerBlock;
    const size_t plane = (size_t)4 * K * C, row = (size_t)2 * C;
    float re[kFftN], im[kFftN];
    {
        const int va = tid / kFftTilesPerBlock, ca = tid % kFftTilesPerBlock;
        const int c = c0 + ca;
        if (va < kFftHalf) {
            const bool ok = c < C;
            const float *src = P + (ok ? c : 0);
#pragma unroll
            for (int u = 0; u < kFftN; ++u) {
                const float *p = src + (size_t)(u * kFftHalf + va) * plane;
                const float rr = ok ? p[(size_t)k * row] : 0.f, ri = ok ? p[(size_t)k * row + C] : 0.f;
                const float ir = ok ? p[(size_t)(K + k) * row] : 0.f, ii = ok ? p[(size_t)(K + k) * row + C] : 0.f;
                re[u] = rr + ii;
                im[u] = ri - ir;
            }
            fft16<1>(re, im);
#pragma unroll
            for (int a = 0; a < kFftN; ++a) {
                sre[(ca * kFftN + a) * kFftHalf + va] = re[a];
                sim[(ca * kFftN + a) * kFftHalf + va] = im[a];
            }
        }
    }
    __syncthreads();
    const int cb = tid / kFftN, ab = tid % kFftN;
    const int c = c0 + cb;
#pragma unroll
    for (int v = 0; v < kFftHalf; ++v) {
        re[v] = sre[(cb * kFftN + ab) * kFftHalf + v];
        im[v] = sim[(cb * kFftN + ab) * kFftHalf + v];
    }
#pragma unroll
    for (int v = kFftHalf; v < kFftN; ++v) {
        re[v] = re[kFftN - v];
        im[v] = -im[kFftN - v];
    }
    fft16<1>(re, im);
    if (c < C && ab < R) {
        float *dst = dw + (((size_t)k * C + c) * R + ab) * S;
#pragma unroll
        for (int s = 0; s < kFftN; ++s)
            if (s < S) {
                const float v = re[s] * (1.f / 256.f);
                dst[s] = beta == 0.f ? v : beta * dst[s] + v;
            }
    }
}

template <class E>
static hipError_t fft_filter_run(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta, float *ws,
                                 hipStream_t s)
{
    const FftGeom gx = fft_geom(d, 0, b);  // x: the Forward input tiles
    FftGeom gd = gx;                        // dy: the output tiles, zero-padded to 16x16
    gd.Ci = d.K; gd.Hi = d.P; gd.Wi = d.Q; gd.pad_h = 0; gd.pad_w = 0;
    gd.win_h = gx.Th; gd.win_w = gx.Tw;
    const int n_tiles = b * gx.T;
    float *Mw = ws;
    float *V = Mw + (size_t)kFftFreqs * 4 * d.K * d.C;
    float *D = V + (size_t)kFftFreqs * 2 * d.C * gx.ld;
    const FastDiv divT(gx.T), divTW(gx.TW);

    LaunchLog *log = launch_log();
    hipError_t e = fill_zero(Mw, (size_t)kFftFreqs * 4 * d.K * d.C, s);
    if (e != hipSuccess) return e;
    const unsigned blocks = (unsigned)((gx.ld + kFftTilesPerBlock - 1) / kFftTilesPerBlock);
    if (log) {
        log->add("fft_input_kernel");
        log->add("fft_input_kernel");
    } else {
        fft_input_kernel<E><<<dim3(blocks, (unsigned)(d.C < 1024 ? d.C : 1024)), kFftThreads, 0, s>>>(x, V, gx, divT, divTW, n_tiles);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        fft_input_kernel<E><<<dim3(blocks, (unsigned)(d.K < 1024 ? d.K : 1024)), kFftThreads, 0, s>>>(dy, D, gd, divT, divTW, n_tiles);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    GemmShape gs{2 * d.K, 2 * d.C, n_tiles};
    gs.batch = kFftFreqs;
    gs.a_batch = (long)2 * d.K * gx.ld;
    gs.b_batch = (long)2 * d.C * gx.ld;
    gs.c_batch = (long)4 * d.K * d.C;
    gs.splits = filter_splits(gs.M, gs.N, gs.Kd, kFftFreqs);
    KLaneParams pa{};
    pa.t = D; pa.bytes = (uint32_t)(gs.a_batch * 4); pa.row_stride = 1; pa.col_stride = gx.ld;
    KLaneParams pb{};
    pb.t = V; pb.bytes = (uint32_t)(gs.b_batch * 4); pb.row_stride = 1; pb.col_stride = gx.ld;
    EpiDenseParams pe{Mw, 2 * d.C};
    if ((e = launch_gemm<KLane0, KLane0, EpiAtomic, true>(pa, pb, pe, gs, s)) != hipSuccess) return e;
    if (log) {
        log->add("fft_dw_kernel");
        return hipSuccess;
    }
    const dim3 go((unsigned)((d.C + kFftTilesPerBlock - 1) / kFftTilesPerBlock), (unsigned)d.K);
    fft_dw_kernel<<<go, kFftThreads, 0, s>>>(Mw, dw, d.K, d.C, d.R, d.S, beta);
    return hipGetLastError();
}

hipError_t fft_bwd_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta, float *ws,
                          hipStream_t s)
{
    return d.dtype == 1 ? fft_filter_run<bf16>(d, b, x, dy, dw, beta, ws, s)
                        : fft_filter_run<float>(d, b, x, dy, dw, beta, ws, s);
}

hipError_t fft_fwd(const Dims &d, int b, const void *x, const void *w, void *y, float *ws, bool filter_ready,
                   hipStream_t s)
{
    return d.dtype == 1 ? fft_run<bf16>(d, 0, b, x, w, y, ws, filter_ready, s)
                        : fft_run<float>(d, 0, b, x, w, y, ws, filter_ready, s);
}

hipError_t fft_bwd_data(const Dims &d, int b, const void *dy, const void *w, void *dx, float *ws, bool filter_ready,
                        hipStream_t s)
{
    return d.dtype == 1 ? fft_run<bf16>(d, 1, b, dy, w, dx, ws, filter_ready, s)
                        : fft_run<float>(d, 1, b, dy, w, dx, ws, filter_ready, s);
}

}  // namespace ucd
