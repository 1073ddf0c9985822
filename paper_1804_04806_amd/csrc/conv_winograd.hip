// Winograd convolution (Lavin & Gray) for 3x3 stride-1 layers, Forward and BackwardData, in two
// sizes: F(2x2,3x3) (4x4 input tiles, 16 products per 2x2 outputs) and F(4x4,3x3) (6x6 input tiles,
// 36 products per 4x4 outputs; interpolation points 0, +-1, +-2, infinity).  With m the output
// tile edge and a = m + 2 the input tile edge, every transform buffer is in the caller's workspace:
//   U[a*a][Ci][Mo4]   filter transform  U = G g G^T            (Mo4 = out channels rounded up to 4)
//   V[a*a][Ci][ld]    input transform   V = B^T d B  per a x a input tile at stride m
//   Z[a*a][Mo][ld]    a*a independent GEMMs  Z_xi = U_xi^T[Mo x Ci] * V_xi[Ci x b*T]   (MFMA)
//   out               output transform  y = A^T z A  per m x m output tile
// with T = ceil(Ho/m) * ceil(Wo/m) tiles per image and ld = b*T rounded up to 4.
// BackwardData is the same pipeline on dy with the filter's two channel indices swapped and its
// taps reversed, and padding 2 - pad.
//
// BackwardFilter is the transposed algorithm F(3x3, m x m): the 3x3 filter gradient of one tile is
// the correlation of its a x a input tile with its m x m tile of dy, and swapping the roles of the
// "filter" and the "output" in the bilinear form gives  dw_tile = G^T [(A dy A^T) . (B^T x B)] G
// with the same three matrices.  The products are summed over all tiles of the micro-batch first:
//   V[a*a][C][ld]     input transform of x, as above
//   D[a*a][K][ld]     D = A dy A^T per m x m tile of dy
//   Mw[a*a][K][C]     a*a GEMMs  Mw_xi = D_xi[K x b*T] * V_xi^T[b*T x C]  (reduction split, atomics)
//   dw                = beta*dw + G^T Mw G per (k, c)
#include <cstdlib>
#include <type_traits>
#include <utility>

#include "gemm_launch.hpp"
#include "kernels.h"

namespace ucd {

// The one-dimensional transforms of F(m,3) (filter, input, output) and of the transposed algorithm
// F(3,m) BackwardFilter uses (grad = A z, filter_t = G^T m); the two-dimensional ones apply them to
// the columns and then to the rows of a tile.
template <int MT>
struct Wino;

template <>
struct Wino<2> {
    static constexpr int A = 4;
    static __device__ __forceinline__ void filter(const float g[3], float u[4])  // G g
    {
        u[0] = g[0];
        u[1] = 0.5f * (g[0] + g[1] + g[2]);
        u[2] = 0.5f * (g[0] - g[1] + g[2]);
        u[3] = g[2];
    }
    static __device__ __forceinline__ void input(const float d[4], float v[4])  // B^T d
    {
        v[0] = d[0] - d[2];
        v[1] = d[1] + d[2];
        v[2] = d[2] - d[1];
        v[3] = d[1] - d[3];
    }
    static __device__ __forceinline__ void output(const float z[4], float y[2])  // A^T z
    {
        y[0] = z[0] + z[1] + z[2];
        y[1] = z[1] - z[2] - z[3];
    }
    static __device__ __forceinline__ void grad(const float z[2], float u[4])  // A z
    {
        u[0] = z[0];
        u[1] = z[0] + z[1];
        u[2] = z[0] - z[1];
        u[3] = -z[1];
    }
    static __device__ __forceinline__ void filter_t(const float m[4], float w[3])  // G^T m
    {
        const float s = 0.5f * (m[1] + m[2]);
        w[0] = m[0] + s;
        w[1] = 0.5f * (m[1] - m[2]);
        w[2] = s + m[3];
    }
};

template <>
struct Wino<4> {
    static constexpr int A = 6;
    static __device__ __forceinline__ void filter(const float g[3], float u[6])
    {
        const float e = g[0] + g[2], f = (1.f / 24.f) * g[0] + (1.f / 6.f) * g[2], h = (1.f / 12.f) * g[1];
        u[0] = 0.25f * g[0];
        u[1] = (-1.f / 6.f) * (e + g[1]);
        u[2] = (-1.f / 6.f) * (e - g[1]);
        u[3] = f + h;
        u[4] = f - h;
        u[5] = g[2];
    }
    static __device__ __forceinline__ void input(const float d[6], float v[6])
    {
        const float a = d[4] - 4.f * d[2], b = d[3] - 4.f * d[1], c = d[4] - d[2], e = 2.f * (d[3] - d[1]);
        v[0] = 4.f * d[0] - 5.f * d[2] + d[4];
        v[1] = a + b;
        v[2] = a - b;
        v[3] = c + e;
        v[4] = c - e;
        v[5] = 4.f * d[1] - 5.f * d[3] + d[5];
    }
    static __device__ __forceinline__ void output(const float z[6], float y[4])
    {
        const float s12 = z[1] + z[2], d12 = z[1] - z[2], s34 = z[3] + z[4], d34 = z[3] - z[4];
        y[0] = z[0] + s12 + s34;
        y[1] = d12 + 2.f * d34;
        y[2] = s12 + 4.f * s34;
        y[3] = d12 + 8.f * d34 + z[5];
    }
    static __device__ __forceinline__ void grad(const float z[4], float u[6])
    {
        const float e = z[0] + z[2], o = z[1] + z[3], e4 = z[0] + 4.f * z[2], o4 = 2.f * z[1] + 8.f * z[3];
        u[0] = z[0];
        u[1] = e + o;
        u[2] = e - o;
        u[3] = e4 + o4;
        u[4] = e4 - o4;
        u[5] = z[3];
    }
    static __device__ __forceinline__ void filter_t(const float m[6], float w[3])
    {
        const float s12 = m[1] + m[2], d12 = m[1] - m[2], s34 = m[3] + m[4], d34 = m[3] - m[4];
        w[0] = 0.25f * m[0] - (1.f / 6.f) * s12 + (1.f / 24.f) * s34;
        w[1] = (-1.f / 6.f) * d12 + (1.f / 12.f) * d34;
        w[2] = (-1.f / 6.f) * s12 + (1.f / 6.f) * s34 + m[5];
    }
};

struct WinoGeom {
    int Ci, Co, Hi, Wi, Ho, Wo, pad_h, pad_w;
    int TH, TW, T;
    int Mo4, ld;
    bool transposed;  // BackwardData: filter read as w[ci][co] with reversed taps
    // strided BackwardData as a stride-1 convolution over dy whose output channels are (c, row phase,
    // column phase): the strides (1, 1 otherwise), and dx's channels, size and the layer's padding
    int sh, sw, oc, oh, ow, oph, opw;
};

// BackwardData of a strided layer, one output phase at a time, is a stride-1 correlation of dy with the
// taps r = phase + stride * i of the filter: with three such taps per axis (11x11 stride 4, 5x5 stride
// 2, 7x7 stride 3, ...) all sh*sw phases together are one 3x3 stride-1 convolution from K channels to
// C*sh*sw, which F(2x2,3x3) computes in 16/(3*3) of the multiplications, followed by a scatter of the
// phases into dx.  (Two taps per axis would cost more than the direct sum, four do not fit 3x3.)
static bool phased_applies(const Dims &d, int op)
{
    if (op != 1 || (d.sh == 1 && d.sw == 1)) return false;
    return (d.R + d.sh - 1) / d.sh == 3 && (d.S + d.sw - 1) / d.sw == 3 && d.ph < d.R && d.pw < d.S;
}

static WinoGeom geom(const Dims &d, int op, int b, int mt)
{
    WinoGeom g;
    g.sh = g.sw = 1; g.oc = g.oh = g.ow = g.oph = g.opw = 0;
    if (phased_applies(d, op)) {
        // dx[c, sh*a + pr - ph, sw*b + pc - pw] = sum_k sum_{i,j < 3} dy[k, a - i, b - j] w[k, c, pr + sh*i, pc + sw*j]:
        // as a correlation over dy padded by 2, output (a, b) in [0, (H-1+ph)/sh] x [0, (W-1+pw)/sw]
        g.Ci = d.K; g.Co = d.C * d.sh * d.sw; g.Hi = d.P; g.Wi = d.Q;
        g.Ho = (d.H - 1 + d.ph) / d.sh + 1; g.Wo = (d.W - 1 + d.pw) / d.sw + 1;
        g.pad_h = g.pad_w = 2; g.transposed = true;
        g.sh = d.sh; g.sw = d.sw; g.oc = d.C; g.oh = d.H; g.ow = d.W; g.oph = d.ph; g.opw = d.pw;
    } else if (op == 0) {
        g.Ci = d.C; g.Co = d.K; g.Hi = d.H; g.Wi = d.W; g.Ho = d.P; g.Wo = d.Q;
        g.pad_h = d.ph; g.pad_w = d.pw; g.transposed = false;
    } else {
        g.Ci = d.K; g.Co = d.C; g.Hi = d.P; g.Wi = d.Q; g.Ho = d.H; g.Wo = d.W;
        g.pad_h = 2 - d.ph; g.pad_w = 2 - d.pw; g.transposed = true;
    }
    g.TH = (g.Ho + mt - 1) / mt; g.TW = (g.Wo + mt - 1) / mt; g.T = g.TH * g.TW;
    g.Mo4 = (g.Co + 3) / 4 * 4;
    g.ld = (b * g.T + 3) / 4 * 4;
    return g;
}

bool winograd_fused_applies(const Dims &d, int op) { return winograd_applies(d, op) || phased_applies(d, op); }

bool winograd_applies(const Dims &d, int op)
{
    if (op < 0 || op > 2) return false;
    if (d.R != 3 || d.S != 3 || d.sh != 1 || d.sw != 1) return false;
    return d.ph <= 2 && d.pw <= 2;
}

size_t winograd_ws_bytes(const Dims &d, int op, int b, int mt)
{
    const size_t planes = (size_t)(mt + 2) * (mt + 2);
    if (op == 2) {  // Mw, V, D
        const WinoGeom g = geom(d, 0, b, mt);
        return 4 * planes * ((size_t)d.K * d.C + (size_t)g.ld * (d.C + d.K));
    }
    const WinoGeom g = geom(d, op, b, mt);
    return 4 * planes * ((size_t)g.Ci * g.Mo4 + (size_t)g.ld * (g.Ci + g.Co));
}

// U[xi][ci][co] = (G g G^T)[xi], one thread per (ci, co) filter; pads co up to Mo4 with zeros.
template <class E, int MT>
__global__ __launch_bounds__(256) void wino_filter_kernel(const void *__restrict__ w, float *__restrict__ U, int Ci,
                                                          int Co, int Mo4, int transposed, int Cpad)
{
    // a plane of U has Cpad >= Ci rows; rows past Ci are written as zeros
    constexpr int A = Wino<MT>::A;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= Cpad * Mo4) return;
    const int ci = i / Mo4, co = i - ci * Mo4;
    float t[A][3];  // G g, column by column
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        float g[3], u[A];
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            float v = 0.f;
            if (co < Co && ci < Ci)
                v = transposed ? Elem<E>::get(w, ((size_t)(ci * Co + co) * 3 + (2 - r)) * 3 + (2 - s))
                               : Elem<E>::get(w, ((size_t)(co * Ci + ci) * 3 + r) * 3 + s);
            g[r] = v;
        }
        Wino<MT>::filter(g, u);
#pragma unroll
        for (int r = 0; r < A; ++r) t[r][s] = u[r];
    }
    const size_t plane = (size_t)Cpad * Mo4;
#pragma unroll
    for (int r = 0; r < A; ++r) {
        float u[A];
        Wino<MT>::filter(t[r], u);
#pragma unroll
        for (int s = 0; s < A; ++s) U[(size_t)(r * A + s) * plane + i] = u[s];
    }
}

// The same for the phases of a strided BackwardData: input channel k, output channel co = (c*sh + pr)*sw + pc,
// taps g[i'][j'] = w[k, c, pr + sh*(2 - i'), pc + sw*(2 - j')] (zero past the filter's end).
template <class E>
__global__ __launch_bounds__(256) void wino_phase_filter_kernel(const void *__restrict__ w, float *__restrict__ U,
                                                                int K, int C, int R, int S, int sh, int sw, int Mo4,
                                                                int Cpad)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= Cpad * Mo4) return;
    const int k = i / Mo4, co = i - k * Mo4;
    const int c = co / (sh * sw), pr = co / sw % sh, pc = co % sw;
    const bool live = k < K && c < C;
    float t[4][3];  // G g, column by column
#pragma unroll
    for (int jj = 0; jj < 3; ++jj) {
        float g[3], u[4];
        const int ss = pc + sw * (2 - jj);
#pragma unroll
        for (int ii = 0; ii < 3; ++ii) {
            const int rr = pr + sh * (2 - ii);
            g[ii] = live && rr < R && ss < S ? Elem<E>::get(w, ((size_t)(k * C + c) * R + rr) * S + ss) : 0.f;
        }
        Wino<2>::filter(g, u);
#pragma unroll
        for (int r = 0; r < 4; ++r) t[r][jj] = u[r];
    }
    const size_t plane = (size_t)Cpad * Mo4;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float u[4];
        Wino<2>::filter(t[r], u);
#pragma unroll
        for (int q = 0; q < 4; ++q) U[(size_t)(r * 4 + q) * plane + i] = u[q];
    }
}

// V[xi][ci][j] for tile j = n*T + th*TW + tw: lanes along j (coalesced plane writes).
template <class E, int MT>
__global__ __launch_bounds__(256) void wino_input_kernel(const void *__restrict__ x, float *__restrict__ V,
                                                         WinoGeom g, FastDiv divT, FastDiv divTW, int n_tiles)
{
    constexpr int A = Wino<MT>::A;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= g.ld) return;
    const size_t plane = (size_t)g.Ci * g.ld;
    uint32_t n = 0, t, th = 0, tw = 0;
    if (j < n_tiles) {
        divT.divmod((uint32_t)j, n, t);
        divTW.divmod(t, th, tw);
    }
    const int h0 = MT * (int)th - g.pad_h, w0 = MT * (int)tw - g.pad_w;
    for (int ci = blockIdx.y; ci < g.Ci; ci += gridDim.y) {
        const size_t src = ((size_t)n * g.Ci + ci) * g.Hi * g.Wi;
        float tr[A][A];  // B^T d, column by column
#pragma unroll
        for (int s = 0; s < A; ++s) {
            float d[A], v[A];
            const int ww = w0 + s;
#pragma unroll
            for (int r = 0; r < A; ++r) {
                const int h = h0 + r;
                d[r] = (j < n_tiles && (unsigned)h < (unsigned)g.Hi && (unsigned)ww < (unsigned)g.Wi)
                           ? Elem<E>::get(x, src + h * g.Wi + ww)
                           : 0.f;
            }
            Wino<MT>::input(d, v);
#pragma unroll
            for (int r = 0; r < A; ++r) tr[r][s] = v[r];
        }
        float *dst = V + (size_t)ci * g.ld + j;
#pragma unroll
        for (int r = 0; r < A; ++r) {
            float v[A];
            Wino<MT>::input(tr[r], v);
#pragma unroll
            for (int s = 0; s < A; ++s) dst[(size_t)(r * A + s) * plane] = v[s];
        }
    }
}

// out[n, co, m*th + {0..m-1}, m*tw + {0..m-1}] = A^T z A, lanes along the tile index.
template <class E, int MT>
__global__ __launch_bounds__(256) void wino_output_kernel(const float *__restrict__ Z, void *__restrict__ out,
                                                          WinoGeom g, FastDiv divT, FastDiv divTW, int n_tiles)
{
    constexpr int A = Wino<MT>::A;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n_tiles) return;
    uint32_t n, t, th, tw;
    divT.divmod((uint32_t)j, n, t);
    divTW.divmod(t, th, tw);
    const int h0 = MT * (int)th, w0 = MT * (int)tw;
    const size_t plane = (size_t)g.Co * g.ld;
    for (int co = blockIdx.y; co < g.Co; co += gridDim.y) {
        const float *src = Z + (size_t)co * g.ld + j;
        float tr[MT][A];  // A^T z, column by column
#pragma unroll
        for (int s = 0; s < A; ++s) {
            float z[A], y[MT];
#pragma unroll
            for (int r = 0; r < A; ++r) z[r] = src[(size_t)(r * A + s) * plane];
            Wino<MT>::output(z, y);
#pragma unroll
            for (int r = 0; r < MT; ++r) tr[r][s] = y[r];
        }
        const size_t dst = ((size_t)n * g.Co + co) * g.Ho * g.Wo;
#pragma unroll
        for (int r = 0; r < MT; ++r) {
            const int h = h0 + r;
            if (h >= g.Ho) continue;
            float y[MT];
            Wino<MT>::output(tr[r], y);
#pragma unroll
            for (int s = 0; s < MT; ++s)
                if (w0 + s < g.Wo) Elem<E>::store(out, dst + h * g.Wo + w0 + s, y[s]);
        }
    }
}

template <class E, int MT>
static hipError_t winograd_run(const Dims &d, int op, int b, const void *in, const void *w, void *out,
                               float *ws, bool filter_ready, hipStream_t s)
{
    constexpr int AA = Wino<MT>::A * Wino<MT>::A;
    const WinoGeom g = geom(d, op, b, MT);
    const int n_tiles = b * g.T;
    float *U = ws;
    float *V = U + (size_t)AA * g.Ci * g.Mo4;
    float *Z = V + (size_t)AA * g.Ci * g.ld;
    const FastDiv divT(g.T), divTW(g.TW);

    LaunchLog *log = launch_log();
    if (filter_ready) {
        // U of this filter is still at the head of the workspace from the previous micro-batch
    } else if (log) log->add("wino_filter_kernel");
    else
        wino_filter_kernel<E, MT><<<(unsigned)((g.Ci * g.Mo4 + 255) / 256), 256, 0, s>>>(w, U, g.Ci, g.Co, g.Mo4,
                                                                                      g.transposed ? 1 : 0, g.Ci);
    hipError_t e = log ? hipSuccess : hipGetLastError();
    if (e != hipSuccess) return e;

    dim3 gi((unsigned)((g.ld + 255) / 256), (unsigned)(g.Ci < 4096 ? g.Ci : 4096));
    if (log) log->add("wino_input_kernel");
    else
        wino_input_kernel<E, MT><<<gi, 256, 0, s>>>(in, V, g, divT, divTW, n_tiles);
    if (!log && (e = hipGetLastError()) != hipSuccess) return e;

    GemmShape gs{g.Co, n_tiles, g.Ci};
    gs.batch = AA;
    gs.a_batch = (long)g.Ci * g.Mo4;
    gs.b_batch = (long)g.Ci * g.ld;
    gs.c_batch = (long)g.Co * g.ld;
    DenseParams pa{U, (uint32_t)(gs.a_batch * 4), g.Mo4};
    DenseParams pb{V, (uint32_t)(gs.b_batch * 4), g.ld};
    EpiDenseParams pe{Z, g.ld};
    if ((e = launch_gemm<DenseNLane, DenseNLane, EpiDense>(pa, pb, pe, gs, s)) != hipSuccess) return e;

    dim3 go((unsigned)((n_tiles + 255) / 256), (unsigned)(g.Co < 4096 ? g.Co : 4096));
    if (log) {
        log->add("wino_output_kernel");
        return hipSuccess;
    }
    wino_output_kernel<E, MT><<<go, 256, 0, s>>>(Z, out, g, divT, divTW, n_tiles);
    return hipGetLastError();
}

// ---- F(2x2,3x3) with both data transforms fused into the GEMM kernel --------------------------------
// The only workspace is the transformed filter U (64*Ci'*Mo4 bytes with Ci' = Ci rounded up to the
// channel step, whatever the micro-batch), so the whole mini-batch can run in one launch under a
// small workspace limit.  A workgroup owns a block of 64 output channels x 64 tiles for all 16
// transform points: each of its four waves keeps 16 accumulator tiles of 32 channels x 32 tiles
// (256 registers, one wave per SIMD).  Per step of kFuC input channels every thread fetches the 4x4
// input patches of kFuC/4 (tile, channel) pairs, transforms them in registers (32 additions each)
// and writes their 16 values to LDS; U's slice for the step is copied from the workspace to LDS
// (rows of channels past Ci are zero there); then 16 points x kFuC/2 channel pairs of MFMAs per
// wave.  After the last channel the 16 accumulators of an (output channel, tile) are combined by
// A^T . A in registers and the 2x2 outputs stored.  Global loads run two steps ahead of the MFMAs
// (one register set, two LDS buffers), and the step's memory and transform work is dealt out behind
// individual MFMAs.
//
// Sixteen 4-byte loads per patch, lanes 8 bytes apart, cost the vector memory pipeline ~34 cache
// accesses per wave instruction (the patch loads of AlexNet conv4 alone keep it busy for half of the
// kernel's time).  PW >= 0 (fp32 tensors, horizontal padding PW = 0 or 1) fetches a patch row with
// one 12- or 16-byte load instead (~21 accesses), starting at column 2*tw (never negative, so no
// address before the tensor is formed): that window holds patch columns PW.. of the row; for PW = 1
// the patch's first column is the second element of the window of the tile to the left, i.e. of
// the lane below (one cross-lane move; lane 0 fetches it with a load of its own, tiles in the
// first tile column take 0).  Window elements past the end of the row belong to the next row and
// are replaced by 0.  PW = -1 is the element-wise form (any padding, bf16).
#ifndef UCD_FUSED_CHANNELS
#define UCD_FUSED_CHANNELS 8
#endif
constexpr int kFuK = 64, kFuT = 64, kFuC = UCD_FUSED_CHANNELS;  // block: channels x tiles; input channels per step
constexpr int kFuNP = kFuC / 4;   // input patches per thread and step (channel = wave + 4h)
constexpr int kFuNU = kFuC;       // float4 pieces of the step's U slice per thread
constexpr int kFuPairs = kFuC / 2;

struct FusedParams {
    const void *in;
    const float *U;
    void *out;
    uint32_t in_bytes, u_bytes;
    WinoGeom g;
    FastDiv divT, divTW;
    int n_tiles, k_blocks;
    int ci_pad;   // rows of a plane of U: Ci rounded up to the channel step
};

template <class E, int PW, bool ODD_W = false, bool PHASED = false, bool WIDE = false>
__global__ __launch_bounds__(256) void wino_fused_kernel(FusedParams p)
{
    constexpr uint32_t EB = Elem<E>::kBytes;
    constexpr bool kRows = PW >= 0;   // row-vector patch loads
    static_assert(!kRows || EB == 4, "row loads are written for fp32 tensors");
    static_assert(!WIDE || kRows, "the wide block is written for row loads");
    // block: 64 output channels x 64 tiles (waves 2 x 2), or WIDE: 128 x 32 (waves 4 x 1).  The wide block
    // transforms one patch per thread and step instead of two (every patch serves twice as many output
    // channels) and reads twice as much of U; LDS: 128 + 32 KB instead of 64 + 64.
    constexpr int KB = WIDE ? 128 : kFuK, TB = WIDE ? 32 : kFuT;
    constexpr int NP = WIDE ? 1 : kFuNP;             // input patches per thread and step
    constexpr int NU = kFuC * 16 * KB / 4 / 256;     // float4 pieces of the step's U slice per thread
    __shared__ __attribute__((aligned(16))) float Us[2][16][kFuC][KB];
    __shared__ __attribute__((aligned(16))) float Vs[2][16][kFuC][TB];
    const WinoGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int wk = WIDE ? wave : wave & 1, wt = WIDE ? 0 : wave >> 1;

    // consecutive work items of an XCD share a tile block (the input patches) and differ in the
    // channel block
    const uint32_t v = xcd_order(blockIdx.x, gridDim.x);
    const int kb = (int)(v % (uint32_t)p.k_blocks), tb = (int)(v / (uint32_t)p.k_blocks);
    const int k0 = kb * KB, t0 = tb * TB;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc_bytes(p.in, 0, p.in_bytes);
    const __amdgpu_buffer_rsrc_t ru = make_rsrc_bytes(p.U, 0, p.u_bytes);

    // producer role: the 4x4 patch of tile `lane` of the block, for channels wave, wave + 4, ... of the step
    // (WIDE: of tile lane % 32, for channel 2 * wave + lane / 32; the upper half's channel is part of its
    // offsets).  The lanes that fetch their own first columns: lane 0, or WIDE the first of every 16
    // (the cross-lane move then stays within rows of 16 lanes).
    const int ptile = WIDE ? l32 : lane;
    const bool own_lane = WIDE ? (lane & 15) == 0 : lane == 0;
    uint32_t voff[kRows ? 4 : 16];   // element-wise: one offset per pixel; rows: the window start of each row
    uint32_t xoff[4];                // rows, PW >= 1: the patch's first PW columns, fetched by lane 0 only
    bool first_col = false, ok1 = true, ok2 = true, ok3 = true;  // rows: tile column 0; window elements inside the row
    bool ok0 = true, okm1 = true, okm2 = true;   // PW = 2: the window's first element and the two columns before it
    {
        const int j = t0 + ptile;
        uint32_t n = 0, t, th = 0, tw = 0;
        const bool live = j < p.n_tiles;
        if (live) {
            p.divT.divmod((uint32_t)j, n, t);
            p.divTW.divmod(t, th, tw);
        }
        const int h0 = 2 * (int)th - g.pad_h, w0 = 2 * (int)tw - g.pad_w;
        const uint32_t half_chan = WIDE ? EB * (uint32_t)(lhi * g.Hi * g.Wi) : 0u;
        if constexpr (kRows) {
            const int ws = 2 * (int)tw;   // = w0 + PW
            first_col = tw == 0;
            ok1 = ws + 1 < g.Wi; ok2 = ws + 2 < g.Wi; ok3 = ws + 3 < g.Wi;
            ok0 = ws < g.Wi; okm1 = ws - 1 < g.Wi; okm2 = ws - 2 < g.Wi;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int h = h0 + r;
                const bool ok = live && (unsigned)h < (unsigned)g.Hi;
                const uint32_t row = EB * (uint32_t)(((int)n * g.Ci * g.Hi + h) * g.Wi + ws) + half_chan;
                voff[r] = ok ? row : kOob;
                xoff[r] = ok && PW >= 1 && own_lane && tw > 0 ? row - PW * EB : kOob;
            }
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int h = h0 + r, w = w0 + c;
                    const bool ok = live && (unsigned)h < (unsigned)g.Hi && (unsigned)w < (unsigned)g.Wi;
                    voff[4 * r + c] = ok ? EB * (uint32_t)(((int)n * g.Ci * g.Hi + h) * g.Wi + w) : kOob;
                }
        }
    }
    // U slice of a step: 16 points x kFuC channels x 64 output channels, as float4: piece id = tid + 256*i
    // -> row = id / 16 = point * kFuC + channel, 4 output channels from 4 * (id % 16)
    uint32_t uoff[NU];
#pragma unroll
    for (int i = 0; i < NU; ++i) {
        const int id = tid + 256 * i, row = id / (KB / 4), q = id % (KB / 4);
        const int xi = row / kFuC, c = row % kFuC, k = k0 + 4 * q;
        uoff[i] = k < g.Mo4 ? 4u * (uint32_t)((xi * p.ci_pad + c) * g.Mo4 + k) : kOob;
    }

    // the thread's input patches of the step after the one in LDS: 16 pixels each, or per row a window
    // of 2 (PW = 2), 3 (PW = 1) or 4 (PW = 0) pixels at the end of d[h][4r..] and, for PW >= 1, lane 0's
    // first PW columns in dx
    float d[NP][16];
    float dx[NP][PW == 2 ? 8 : 4];
    f32x4 uq[NU];        // and its share of that step's U slice
    // a channel past the last one gets a scalar offset that pushes every address out of range
    auto chan_off = [&](int c0, int h) {
        // WIDE: the lower half's channel; the upper half's, one further, may be the first one past the
        // last: it then reads the next image's data (or nothing), and U's rows past Ci are zero
        const int c = WIDE ? c0 + 2 * wave : c0 + wave + 4 * h;
        return c < g.Ci ? EB * (uint32_t)(c * g.Hi * g.Wi) : kOob;
    };
    constexpr int kPatchLoads = !kRows ? 16 : PW >= 1 ? 8 : 4;   // load instructions per patch
    auto fetch_piece = [&](int c0, int h, int i) {   // i < kPatchLoads
        const uint32_t so = chan_off(c0, h);
        if constexpr (!kRows) {
            d[h][i] = Elem<E>::load(rin, voff[i], so);
        } else if constexpr (PW == 0) {
            const f32x4 q = buf_load4(rin, voff[i], so);
            d[h][4 * i] = q.x; d[h][4 * i + 1] = q.y; d[h][4 * i + 2] = q.z; d[h][4 * i + 3] = q.w;
        } else if constexpr (PW == 2) {
            if (i < 4) {
                const auto q = __builtin_amdgcn_raw_buffer_load_b64(rin, (int)voff[i], (int)so, 0);
                d[h][4 * i + 2] = __uint_as_float(q[0]); d[h][4 * i + 3] = __uint_as_float(q[1]);
            } else {
                const auto q = __builtin_amdgcn_raw_buffer_load_b64(rin, (int)xoff[i - 4], (int)so, 0);
                dx[h][2 * (i - 4)] = __uint_as_float(q[0]); dx[h][2 * (i - 4) + 1] = __uint_as_float(q[1]);
            }
        } else if (i < 4) {
            const auto q = __builtin_amdgcn_raw_buffer_load_b96(rin, (int)voff[i], (int)so, 0);
#pragma unroll
            for (int c = 0; c < 3; ++c) d[h][4 * i + 1 + c] = __uint_as_float(q[c]);
        } else {
            dx[h][i - 4] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rin, (int)xoff[i - 4], (int)so, 0));
        }
    };
    auto fetch_patch = [&](int c0, int h) {
#pragma unroll
        for (int i = 0; i < kPatchLoads; ++i) fetch_piece(c0, h, i);
    };
    // rows: the windows as loaded become the patch (first column from the lane below, zeros outside the row)
    constexpr int kShr = WIDE ? 0x111 : 0x138;   // row_shr:1 (rows of 16 lanes) | wave_shr:1
    auto finish_patch = [&](int h) {
        if constexpr (kRows) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (PW == 1) {
                    // Window = columns 2tw, 2tw+1, 2tw+2.  With an even width only the last one can lie
                    // past the row (in the last tile column); with an odd width the last two can, and
                    // the tile to the left of a first-column tile is then a last-column tile whose
                    // second window element has just been zeroed: the cross-lane move delivers the 0.
                    if constexpr (ODD_W) d[h][4 * r + 2] = ok1 ? d[h][4 * r + 2] : 0.f;
                    d[h][4 * r + 3] = ok2 ? d[h][4 * r + 3] : 0.f;
                    // every lane takes the value of the lane below; the lanes that loaded their own keep `old`
                    const int left = __builtin_amdgcn_update_dpp((int)__float_as_uint(dx[h][r]),
                                                                 (int)__float_as_uint(d[h][4 * r + 2]), kShr, 0xf, 0xf, false);
                    d[h][4 * r] = ODD_W ? __uint_as_float((uint32_t)left) : first_col ? 0.f : __uint_as_float((uint32_t)left);
                } else if constexpr (PW == 2) {
                    // Window = columns 2tw, 2tw+1 = patch columns 2, 3; the last tile column's window can
                    // lie past the row altogether.  Patch columns 0, 1 are the window of the tile to the
                    // left, already masked there (lane 0: its own load, whose second element can be past
                    // the row when the width is odd, and both when the output is more than two columns
                    // wider than the input, as the phase form of a strided BackwardData can be); zeros in
                    // the first tile column.
                    d[h][4 * r + 2] = ok0 ? d[h][4 * r + 2] : 0.f;
                    d[h][4 * r + 3] = ok1 ? d[h][4 * r + 3] : 0.f;
                    const float own0 = okm2 ? dx[h][2 * r] : 0.f;
                    const float own1 = okm1 ? dx[h][2 * r + 1] : 0.f;
                    const int l0 = __builtin_amdgcn_update_dpp((int)__float_as_uint(own0),
                                                               (int)__float_as_uint(d[h][4 * r + 2]), kShr, 0xf, 0xf, false);
                    const int l1 = __builtin_amdgcn_update_dpp((int)__float_as_uint(own1),
                                                               (int)__float_as_uint(d[h][4 * r + 3]), kShr, 0xf, 0xf, false);
                    d[h][4 * r] = first_col ? 0.f : __uint_as_float((uint32_t)l0);
                    d[h][4 * r + 1] = first_col ? 0.f : __uint_as_float((uint32_t)l1);
                } else {
                    d[h][4 * r + 1] = ok1 ? d[h][4 * r + 1] : 0.f;
                    d[h][4 * r + 2] = ok2 ? d[h][4 * r + 2] : 0.f;
                    d[h][4 * r + 3] = ok3 ? d[h][4 * r + 3] : 0.f;
                }
            }
        }
    };
    // U's planes have ci_pad rows (zero past Ci), so every step is whole and its part of the address is
    // a scalar offset; a load for a step past the last one reads the next point's rows or out of range
    // and is never used
    auto fetch_u = [&](int c0, int i) { uq[i] = buf_load4(ru, uoff[i], 4u * (uint32_t)(c0 * g.Mo4)); };
    // B^T d B of patch h into LDS buffer `buf`: points 4r .. 4r+3 from row r of B^T d
    auto vrow = [&](int h) { return WIDE ? 2 * wave + lhi : wave + 4 * h; };
    auto store_v = [&](int buf, int h) {
        finish_patch(h);
        float tr[16];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float a0 = d[h][c], a1 = d[h][4 + c], a2 = d[h][8 + c], a3 = d[h][12 + c];
            tr[c] = a0 - a2;
            tr[4 + c] = a1 + a2;
            tr[8 + c] = a2 - a1;
            tr[12 + c] = a1 - a3;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float a0 = tr[4 * r], a1 = tr[4 * r + 1], a2 = tr[4 * r + 2], a3 = tr[4 * r + 3];
            Vs[buf][4 * r + 0][vrow(h)][ptile] = a0 - a2;
            Vs[buf][4 * r + 1][vrow(h)][ptile] = a1 + a2;
            Vs[buf][4 * r + 2][vrow(h)][ptile] = a2 - a1;
            Vs[buf][4 * r + 3][vrow(h)][ptile] = a1 - a3;
        }
    };
    // piece i goes to row (tid >> 4) + 16 i of the buffer's [16 * kFuC][64] slab: one address per
    // thread, the pieces 1024 floats apart (immediate offsets)
    const int u_slot = 4 * tid;
    auto store_u = [&](int buf, int i) {
        *reinterpret_cast<f32x4 *>(&Us[buf][0][0][0] + u_slot + 1024 * i) = uq[i];
    };

    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

#pragma unroll
    for (int h = 0; h < NP; ++h) fetch_patch(0, h);
#pragma unroll
    for (int i = 0; i < NU; ++i) fetch_u(0, i);
#pragma unroll
    for (int h = 0; h < NP; ++h) store_v(0, h);
#pragma unroll
    for (int i = 0; i < NU; ++i) store_u(0, i);
#pragma unroll
    for (int h = 0; h < NP; ++h) fetch_patch(kFuC, h);
#pragma unroll
    for (int i = 0; i < NU; ++i) fetch_u(kFuC, i);
    __syncthreads();

    int buf = 0;
    for (int c0 = 0; c0 < g.Ci; c0 += kFuC) {
        const float *ua = &Us[buf][0][lhi][wk * 32 + l32];
        const float *vb = &Vs[buf][0][lhi][wt * 32 + l32];
        // Operands of (point xi, channel pair q): rows 2q + lhi of the point's slab.  They are read in
        // units of two channel pairs (one two-address LDS read per operand), kAhead units before the
        // unit's MFMAs: four units of registers, one in use, three on their way.
        constexpr int kUnits = 16 * kFuPairs / 2, kAhead = 3;
        float a[kAhead + 1][2], b[kAhead + 1][2];
        auto read_unit = [&](int u) {
            const int xi = u / (kFuPairs / 2), q0 = 2 * (u % (kFuPairs / 2));
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                a[u % (kAhead + 1)][q] = ua[(xi * kFuC + 2 * (q0 + q)) * KB];
                b[u % (kAhead + 1)][q] = vb[(xi * kFuC + 2 * (q0 + q)) * TB];
            }
        };
#pragma unroll
        for (int u = 0; u < kAhead; ++u) read_unit(u);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(UCD_MFMA_PRIO);
        constexpr int kMfmas = 16 * kFuPairs;
        // One MFMA and what is dealt out behind it; m is a compile-time constant so that every slot
        // holds its own piece of work only (a loop left to the unroller keeps all pieces in every
        // iteration until it has unrolled, and gives up on a body of that size).
        auto slot = [&](auto M) {
            constexpr int m = decltype(M)::value;
            constexpr int xi = m / kFuPairs, u = m / 2;
            acc[xi] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u % (kAhead + 1)][m % 2], b[u % (kAhead + 1)][m % 2], acc[xi], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (m % 2 == 0 && u + kAhead < kUnits) read_unit(u + kAhead);
            // The registers hold step c0 + kFuC as loaded: it is transformed into the other LDS buffer
            // and every register reloaded, as soon as it is free, with step c0 + 2 kFuC.  One piece of
            // that work behind each MFMA, and never more than one global load: a burst of loads blocks
            // the wave at the memory pipeline's queue, and with one wave per SIMD nothing else would
            // feed the matrix pipe meanwhile.
            constexpr int kPatchSlots = 1 + kPatchLoads;  // 1 transform + the patch's loads
            if constexpr (m >= 1 && m < 1 + kPatchSlots * NP) {
                constexpr int h = (m - 1) / kPatchSlots, i = (m - 1) % kPatchSlots;
                if constexpr (i == 0) store_v(buf ^ 1, h);
                else fetch_piece(c0 + 2 * kFuC, h, i - 1);
            }
            constexpr int kUStart = 1 + kPatchSlots * NP;
            if constexpr (m >= kUStart && m < kUStart + 2 * NU) {
                constexpr int i = (m - kUStart) / 2;
                if constexpr ((m - kUStart) % 2 == 0) store_u(buf ^ 1, i);
                else fetch_u(c0 + 2 * kFuC, i);
            }
            static_assert(kUStart + 2 * NU <= 16 * kFuPairs, "the step's work fits behind its MFMAs");
            __builtin_amdgcn_sched_barrier(0);
        };
        static_for<kMfmas>(slot);
        __builtin_amdgcn_s_setprio(0);
        __syncthreads();
        buf ^= 1;
    }

    // output transform and store: lane = tile (column l32 of the wave's 32), register e = channel row
    const int j = t0 + wt * 32 + l32;
    if (j >= p.n_tiles) return;
    uint32_t n, t, th, tw;
    p.divT.divmod((uint32_t)j, n, t);
    p.divTW.divmod(t, th, tw);
    const int h0 = 2 * (int)th, w0 = 2 * (int)tw;
    const bool h1 = h0 + 1 < g.Ho, w1 = w0 + 1 < g.Wo;
    if constexpr (PHASED) {
        // channel k is (c, pr, pc) = ((k / sw) / sh, (k / sw) % sh, k % sw): position (a, b) of the tile goes
        // to dx[c, sh*a + pr - ph, sw*b + pc - pw].  With a column stride of 4 the lane's registers
        // 4q .. 4q+3 are the four column phases of one (c, pr), i.e. four adjacent pixels of dx: one
        // 16-byte store (dword-aligned) unless the four straddle the row's ends.
        typedef float f32x4_dw __attribute__((ext_vector_type(4), aligned(4)));
        const bool quads = EB == 4 && g.sw == 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int kq = k0 + wk * 32 + 8 * q + 4 * lhi;
            float o[4][2][2];   // [register of the quad][row of the tile][column of the tile]
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = 4 * q + i;
                float y[2][4];  // A^T m, column by column
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float m0 = acc[c][e], m1 = acc[4 + c][e], m2 = acc[8 + c][e], m3 = acc[12 + c][e];
                    y[0][c] = m0 + m1 + m2;
                    y[1][c] = m1 - m2 - m3;
                }
#pragma unroll
                for (int dr = 0; dr < 2; ++dr) {
                    o[i][dr][0] = y[dr][0] + y[dr][1] + y[dr][2];
                    o[i][dr][1] = y[dr][1] - y[dr][2] - y[dr][3];
                }
            }
            if (quads) {
                if (kq >= g.Co) continue;
                const int c = kq / (4 * g.sh), pr = kq / 4 % g.sh;
#pragma unroll
                for (int dr = 0; dr < 2; ++dr)
#pragma unroll
                    for (int dc = 0; dc < 2; ++dc) {
                        const int h = g.sh * (h0 + dr) + pr - g.oph, w = 4 * (w0 + dc) - g.opw;
                        if ((unsigned)h >= (unsigned)g.oh) continue;
                        float *dst = (float *)p.out + (((long)n * g.oc + c) * g.oh + h) * g.ow + w;
                        if (w >= 0 && w + 3 < g.ow) {
                            f32x4_dw v4;
                            v4.x = o[0][dr][dc]; v4.y = o[1][dr][dc]; v4.z = o[2][dr][dc]; v4.w = o[3][dr][dc];
                            *reinterpret_cast<f32x4_dw *>(dst) = v4;
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                if ((unsigned)(w + i) < (unsigned)g.ow) dst[i] = o[i][dr][dc];
                        }
                    }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int k = kq + i;
                    if (k >= g.Co) continue;
                    const int c = k / (g.sh * g.sw), pr = k / g.sw % g.sh, pc = k % g.sw;
#pragma unroll
                    for (int dr = 0; dr < 2; ++dr)
#pragma unroll
                        for (int dc = 0; dc < 2; ++dc) {
                            const int h = g.sh * (h0 + dr) + pr - g.oph, w = g.sw * (w0 + dc) + pc - g.opw;
                            if ((unsigned)h < (unsigned)g.oh && (unsigned)w < (unsigned)g.ow)
                                Elem<E>::store(p.out, (((long)n * g.oc + c) * g.oh + h) * g.ow + w, o[i][dr][dc]);
                        }
                }
            }
        }
        return;
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int k = k0 + wk * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
        if (k >= g.Co) continue;
        float y[2][4];  // A^T m, column by column
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float m0 = acc[c][e], m1 = acc[4 + c][e], m2 = acc[8 + c][e], m3 = acc[12 + c][e];
            y[0][c] = m0 + m1 + m2;
            y[1][c] = m1 - m2 - m3;
        }
        const long base = (((long)n * g.Co + k) * g.Ho + h0) * g.Wo + w0;
        Elem<E>::store(p.out, base, y[0][0] + y[0][1] + y[0][2]);
        if (w1) Elem<E>::store(p.out, base + 1, y[0][1] - y[0][2] - y[0][3]);
        if (h1) {
            Elem<E>::store(p.out, base + g.Wo, y[1][0] + y[1][1] + y[1][2]);
            if (w1) Elem<E>::store(p.out, base + g.Wo + 1, y[1][1] - y[1][2] - y[1][3]);
        }
    }
}

// ---- the same on the bf16 matrix pipe (bf16 tensors) ---------------------------------------------
// The transforms run in fp32 as above; U = G g G^T and V = B^T d B are then rounded to bf16 and
// multiplied by v_mfma_f32_32x32x16_bf16 with fp32 accumulation: a step of 16 input channels is one
// MFMA per point and 32x32 tile, an eighth of the fp32 kernel's matrix time, so the kernel lives on
// its vector instructions (unpacking, transforms, packing), its LDS traffic and its loads.  Those
// overlap only between waves, so the workgroup has eight: wave (ph, wk, wt) accumulates the points
// 8*ph .. 8*ph+7 (rows 2*ph, 2*ph+1 of the point grid) of the 32x32 tile (wk, wt) in 128 registers,
// which leaves room for two waves per SIMD; the two halves of a tile's points meet in the output
// transform through LDS.
// LDS and the transformed filter in the workspace hold pairs of consecutive input channels as dwords,
// [point][channel pair][64 rows]: the four pairs of a half-step are the MFMA operand of the lane that
// owns the row (lanes 0-31 pairs 0-3 of the step, lanes 32-63 pairs 4-7), and a wave's accesses are
// consecutive dwords.
// A patch row (4 pixels = 8 bytes at any 2-byte alignment) is fetched as the three aligned dwords that
// cover it and shifted into place by the parity of its first element; pixels outside the row are
// dropped by the byte selectors that widen bf16 to fp32.
constexpr int kBfC = 16;   // input channels per step
constexpr int kBfNU = 4;   // 16-byte pieces of the step's U slice per thread: 16 points x 8 pairs x 64 / 4 / 512

struct FusedBf16Params {
    const void *in;    // the input tensor's address rounded down to 4 bytes
    const void *U;
    void *out;
    uint32_t in_bytes, u_bytes;
    WinoGeom g;
    FastDiv divT, divTW;
    int n_tiles, k_blocks, ci_pad;
    int lead;          // elements between `in` and the tensor's first element: 0 or 1
};

// U as bf16: [point][ci / 2][co (Mo4 rows)][ci % 2], ci padded to Cpad (a multiple of 16) with zeros
template <class E>
__global__ __launch_bounds__(256) void wino_filter_bf16_kernel(const void *__restrict__ w, uint16_t *__restrict__ U,
                                                               int Ci, int Co, int Mo4, int transposed, int Cpad)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= Cpad * Mo4) return;
    const int ci = i / Mo4, co = i - ci * Mo4;
    float t[4][3];  // G g, column by column
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        float g[3], u[4];
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            float v = 0.f;
            if (co < Co && ci < Ci)
                v = transposed ? Elem<E>::get(w, ((size_t)(ci * Co + co) * 3 + (2 - r)) * 3 + (2 - s))
                               : Elem<E>::get(w, ((size_t)(co * Ci + ci) * 3 + r) * 3 + s);
            g[r] = v;
        }
        Wino<2>::filter(g, u);
#pragma unroll
        for (int r = 0; r < 4; ++r) t[r][s] = u[r];
    }
    const size_t plane = (size_t)Cpad * Mo4;   // elements per point
    const size_t at = ((size_t)(ci / 2) * Mo4 + co) * 2 + ci % 2;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float u[4];
        Wino<2>::filter(t[r], u);
#pragma unroll
        for (int q = 0; q < 4; ++q) U[(size_t)(r * 4 + q) * plane + at] = Elem<bf16>::round(u[q]);
    }
}

// The same for the output phases of a strided BackwardData (see wino_phase_filter_kernel): input channel k,
// output channel co = (c*sh + pr)*sw + pc, taps g[i'][j'] = w[k, c, pr + sh*(2 - i'), pc + sw*(2 - j')]
template <class E>
__global__ __launch_bounds__(256) void wino_phase_filter_bf16_kernel(const void *__restrict__ w, uint16_t *__restrict__ U,
                                                                     int K, int C, int R, int S, int sh, int sw, int Mo4,
                                                                     int Cpad)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= Cpad * Mo4) return;
    const int k = i / Mo4, co = i - k * Mo4;
    const int c = co / (sh * sw), pr = co / sw % sh, pc = co % sw;
    const bool live = k < K && c < C;
    float t[4][3];  // G g, column by column
#pragma unroll
    for (int jj = 0; jj < 3; ++jj) {
        float g[3], u[4];
        const int ss = pc + sw * (2 - jj);
#pragma unroll
        for (int ii = 0; ii < 3; ++ii) {
            const int rr = pr + sh * (2 - ii);
            g[ii] = live && rr < R && ss < S ? Elem<E>::get(w, ((size_t)(k * C + c) * R + rr) * S + ss) : 0.f;
        }
        Wino<2>::filter(g, u);
#pragma unroll
        for (int r = 0; r < 4; ++r) t[r][jj] = u[r];
    }
    const size_t plane = (size_t)Cpad * Mo4;
    const size_t at = ((size_t)(k / 2) * Mo4 + co) * 2 + k % 2;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float u[4];
        Wino<2>::filter(t[r], u);
#pragma unroll
        for (int q = 0; q < 4; ++q) U[(size_t)(r * 4 + q) * plane + at] = Elem<bf16>::round(u[q]);
    }
}

template <bool PHASED>
__global__ __launch_bounds__(512) void wino_fused_bf16_kernel(FusedBf16Params p)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef unsigned int u32x3 __attribute__((ext_vector_type(3)));
    // [buffer][point][channel pair of the step][row]: bf16 pairs
    __shared__ __attribute__((aligned(16))) uint32_t Us[2][16][8][64];
    __shared__ __attribute__((aligned(16))) uint32_t Vs[2][16][8][64];
    const WinoGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int ph = wave >> 2, wk = wave & 1, wt = (wave >> 1) & 1;

    const uint32_t v = xcd_order(blockIdx.x, gridDim.x);
    const int kb = (int)(v % (uint32_t)p.k_blocks), tb = (int)(v / (uint32_t)p.k_blocks);
    const int k0 = kb * kFuK, t0 = tb * kFuT;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc_bytes(p.in, 0, p.in_bytes);
    const __amdgpu_buffer_rsrc_t ru = make_rsrc_bytes(p.U, 0, p.u_bytes);

    // producer role: the 4x4 patch of tile `lane` of the block, for channels 2*wave, 2*wave+1 of the step
    // (one channel pair).  Element index of a row's first pixel = lead + c*Hi*Wi + eo[r]; with q = parity
    // of (lead + c*Hi*Wi) the row starts in the dword at element ((eo + q) & ~1) past the channel's
    // dword-aligned base, at its upper half if (eo + q) is odd.  Offsets carry 4 bytes more than that
    // (eo >= -2, so they are never negative) and the channel's scalar offset 4 bytes less.
    uint32_t voffb0[4], voffb1[4];   // per row, for q = 0 and q = 1
    uint32_t sh0[4];        // 16 * parity of eo[row]: the shift for q = 0; for q = 1 the other one
    uint32_t sel[4];        // per patch column: selector that widens the pixel's half of a dword, or zeroes it
    {
        const int j = t0 + lane;
        uint32_t n = 0, t, th = 0, tw = 0;
        const bool live = j < p.n_tiles;
        if (live) {
            p.divT.divmod((uint32_t)j, n, t);
            p.divTW.divmod(t, th, tw);
        }
        const int h0 = 2 * (int)th - g.pad_h, w0 = 2 * (int)tw - g.pad_w;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int h = h0 + r;
            const bool ok = live && (unsigned)h < (unsigned)g.Hi;
            const int eo = ((int)n * g.Ci * g.Hi + h) * g.Wi + w0;
            voffb0[r] = ok ? (uint32_t)(2 * (eo & ~1) + 4) : kOob;
            voffb1[r] = ok ? (uint32_t)(2 * ((eo + 1) & ~1) + 4) : kOob;
            sh0[r] = (uint32_t)(eo & 1) << 4;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c)
            sel[c] = (unsigned)(w0 + c) < (unsigned)g.Wi ? (c & 1 ? 0x03020c0cu : 0x01000c0cu) : 0x0c0c0c0cu;
    }
    const int hw = g.Hi * g.Wi;
    // channel c: the parity q and the scalar byte offset of its loads
    auto chan_q = [&](int c) { return (p.lead + c * hw) & 1; };
    auto chan_soff = [&](int c) {
        if (c >= g.Ci) return kOob;   // past the last channel: every address out of range
        const int base = p.lead + c * hw;
        return (uint32_t)(2 * (base - (base & 1)));   // 4 less is taken off below, where it cannot go negative
    };

    // U slice of a step: piece id = tid + 512*i -> row = id / 16 = point * 8 + pair, output channels 4 * (id % 16) ..+3
    uint32_t uoff[kBfNU];
    const int cpairs = p.ci_pad / 2;
#pragma unroll
    for (int i = 0; i < kBfNU; ++i) {
        const int id = tid + 512 * i, row = id >> 4, k = k0 + 4 * (id & 15);
        const int xi = row >> 3, pair = row & 7;
        uoff[i] = k < g.Mo4 ? 4u * (uint32_t)((xi * cpairs + pair) * g.Mo4 + k) : kOob;
    }

    u32x3 raw[2][4];     // the thread's two patches of the step after the one in LDS, as loaded: [channel][row]
    u32x4 uq[kBfNU];     // and its share of that step's U slice
    auto fetch_row = [&](int c0, int i, int r) {
        const int c = c0 + 2 * wave + i;
        const int q = chan_q(c);
        uint32_t vo = q ? voffb1[r] : voffb0[r];
        uint32_t so = chan_soff(c);
        if (c == 0) {
            // the first channel has no room below its base for the 4 extra bytes: take them off the
            // lane's offset instead; a row that starts before the tensor (first row, first tile column,
            // padded) is fetched from the tensor's start and moved up one dword when it is unpacked
            vo = vo < 4u ? 0u : vo - 4u;
        } else if (so != kOob) {
            so -= 4u;
        }
        raw[i][r] = __builtin_amdgcn_raw_buffer_load_b96(rin, (int)vo, (int)so, 0);
    };
    auto fetch_u = [&](int c0, int i) {
        uq[i] = __builtin_amdgcn_raw_buffer_load_b128(ru, (int)uoff[i], (int)(4u * (uint32_t)((c0 >> 1) * g.Mo4)), 0);
    };
    auto store_u = [&](int buf, int i) {
        *reinterpret_cast<u32x4 *>(&Us[buf][0][0][0] + 4 * (tid + 512 * i)) = uq[i];
    };

    // B^T d B of the two patches, rounded to bf16 and paired
    float vprev[16];   // the transformed patch of the even channel, waiting for its odd partner
    auto transform = [&](int c0, auto I, int buf) {
        constexpr int i = decltype(I)::value;
        const int c = c0 + 2 * wave + i;
        const uint32_t qs = (uint32_t)chan_q(c) << 4;
        float d[16];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            uint32_t d0 = raw[i][r].x, d1 = raw[i][r].y, d2 = raw[i][r].z;
            if (c == 0) {
                const uint32_t vo = chan_q(0) ? voffb1[r] : voffb0[r];
                if (vo < 4u) { d2 = d1; d1 = d0; d0 = 0u; }
            }
            const uint32_t sh = sh0[r] ^ qs;
            const uint32_t w0 = __builtin_amdgcn_alignbit(d1, d0, sh), w1 = __builtin_amdgcn_alignbit(d2, d1, sh);
            d[4 * r + 0] = __uint_as_float(__builtin_amdgcn_perm(0u, w0, sel[0]));
            d[4 * r + 1] = __uint_as_float(__builtin_amdgcn_perm(0u, w0, sel[1]));
            d[4 * r + 2] = __uint_as_float(__builtin_amdgcn_perm(0u, w1, sel[2]));
            d[4 * r + 3] = __uint_as_float(__builtin_amdgcn_perm(0u, w1, sel[3]));
        }
        float tr[16], vv[16];
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const float a0 = d[cc], a1 = d[4 + cc], a2 = d[8 + cc], a3 = d[12 + cc];
            tr[cc] = a0 - a2;
            tr[4 + cc] = a1 + a2;
            tr[8 + cc] = a2 - a1;
            tr[12 + cc] = a1 - a3;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float a0 = tr[4 * r], a1 = tr[4 * r + 1], a2 = tr[4 * r + 2], a3 = tr[4 * r + 3];
            vv[4 * r + 0] = a0 - a2;
            vv[4 * r + 1] = a1 + a2;
            vv[4 * r + 2] = a2 - a1;
            vv[4 * r + 3] = a1 - a3;
        }
        if constexpr (i == 0) {
#pragma unroll
            for (int xi = 0; xi < 16; ++xi) vprev[xi] = vv[xi];
        } else {
            // the thread's channel pair is dword [xi][wave][lane] of the step's slab
#pragma unroll
            for (int xi = 0; xi < 16; ++xi) {
                const f32x2 two = {vprev[xi], vv[xi]};
                const bf16x2 h2 = __builtin_convertvector(two, bf16x2);
                Vs[buf][xi][wave][lane] = *reinterpret_cast<const uint32_t *>(&h2);
            }
        }
    };

    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

    // step 0 -> LDS buffer 0, step 1 -> registers
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) fetch_row(0, i, r);
#pragma unroll
    for (int i = 0; i < kBfNU; ++i) fetch_u(0, i);
    transform(0, std::integral_constant<int, 0>{}, 0);
    transform(0, std::integral_constant<int, 1>{}, 0);
#pragma unroll
    for (int i = 0; i < kBfNU; ++i) store_u(0, i);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) fetch_row(kBfC, i, r);
#pragma unroll
    for (int i = 0; i < kBfNU; ++i) fetch_u(kBfC, i);
    __syncthreads();

    int buf = 0;
    for (int c0 = 0; c0 < g.Ci; c0 += kBfC) {
        // operands of point xi: the lane's row of pairs 4*lhi .. 4*lhi+3
        const uint32_t *ua = &Us[buf][8 * ph][4 * lhi][wk * 32 + l32];
        const uint32_t *vb = &Vs[buf][8 * ph][4 * lhi][wt * 32 + l32];
        u32x4 a[2], b[2];
        auto read_ops = [&](int m) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                a[m & 1][q] = ua[(m * 8 + q) * 64];
                b[m & 1][q] = vb[(m * 8 + q) * 64];
            }
        };
        read_ops(0);
        // one MFMA per point and, behind it, a piece of the next step's work: the registers hold step
        // c0 + 16 as loaded; each patch is transformed and its registers reloaded with step c0 + 32
        auto slot = [&](auto M) {
            constexpr int m = decltype(M)::value;
            if constexpr (m + 1 < 8) read_ops(m + 1);
            acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[m & 1]),
                                                             __builtin_bit_cast(bf16x8, b[m & 1]), acc[m], 0, 0, 0);
            if constexpr (m == 0 || m == 2) {
                transform(c0 + kBfC, std::integral_constant<int, m / 2>{}, buf ^ 1);
            } else if constexpr (m == 1 || m == 3) {
#pragma unroll
                for (int r = 0; r < 4; ++r) fetch_row(c0 + 2 * kBfC, m / 2, r);
            } else if constexpr (m < 6) {
                constexpr int i0 = 2 * (m - 4);
                store_u(buf ^ 1, i0);
                store_u(buf ^ 1, i0 + 1);
                fetch_u(c0 + 2 * kBfC, i0);
                fetch_u(c0 + 2 * kBfC, i0 + 1);
            }
        };
        static_for<8>(slot);
        __syncthreads();
        buf ^= 1;
    }

    // Output transform Y = A^T M A, A^T = [1 1 1 0; 0 1 -1 -1]: this wave holds rows 2*ph, 2*ph+1 of M.
    // Each half forms its share of both output rows; the share of the row it does not store goes to
    // the other half through LDS (the operand buffers are free now), [value][wave][lane].
    float *xch = reinterpret_cast<float *>(&Us[0][0][0][0]);   // 32 values x 8 waves x 64 lanes = 64 KB
    float mine[16][2];   // the row this half stores: ph = 0 the tile's first row, ph = 1 its second
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        // rows ra = M[2ph], rb = M[2ph+1], each times A: two values
        const float a0 = acc[0][e], a1 = acc[1][e], a2 = acc[2][e], a3 = acc[3][e];
        const float b0 = acc[4][e], b1 = acc[5][e], b2 = acc[6][e], b3 = acc[7][e];
        const float ra0 = a0 + a1 + a2, ra1 = a1 - a2 - a3, rb0 = b0 + b1 + b2, rb1 = b1 - b2 - b3;
        // ph = 0: rows 0, 1 of M: Y[0] += ra + rb, Y[1] += rb.   ph = 1: rows 2, 3: Y[0] += ra, Y[1] += -ra - rb
        float keep0, keep1, give0, give1;
        if (ph == 0) { keep0 = ra0 + rb0; keep1 = ra1 + rb1; give0 = rb0; give1 = rb1; }
        else { keep0 = -ra0 - rb0; keep1 = -ra1 - rb1; give0 = ra0; give1 = ra1; }
        mine[e][0] = keep0; mine[e][1] = keep1;
        xch[((2 * e) * 8 + wave) * 64 + lane] = give0;
        xch[((2 * e + 1) * 8 + wave) * 64 + lane] = give1;
    }
    __syncthreads();
    const int j = t0 + wt * 32 + l32;
    if (j >= p.n_tiles) return;
    uint32_t n, t, th, tw;
    p.divT.divmod((uint32_t)j, n, t);
    p.divTW.divmod(t, th, tw);
    const int ho = 2 * (int)th + ph, wo = 2 * (int)tw;
    if (ho >= g.Ho) return;
    const bool w1 = wo + 1 < g.Wo;
    const int other = wave ^ 4;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int k = k0 + wk * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
        if (k >= g.Co) continue;
        const float y0 = mine[e][0] + xch[((2 * e) * 8 + other) * 64 + lane];
        const float y1 = mine[e][1] + xch[((2 * e + 1) * 8 + other) * 64 + lane];
        if constexpr (PHASED) {
            // channel k is (c, pr, pc): position (a, b) of the tile goes to dx[c, sh*a + pr - ph, sw*b + pc - pw]
            const int c = k / (g.sh * g.sw), pr = k / g.sw % g.sh, pc = k % g.sw;
            const int h = g.sh * ho + pr - g.oph;
            if ((unsigned)h >= (unsigned)g.oh) continue;
            const long row = (((long)n * g.oc + c) * g.oh + h) * g.ow;
            const int wa = g.sw * wo + pc - g.opw, wb = wa + g.sw;
            if ((unsigned)wa < (unsigned)g.ow) Elem<bf16>::store(p.out, row + wa, y0);
            if (w1 && (unsigned)wb < (unsigned)g.ow) Elem<bf16>::store(p.out, row + wb, y1);
            continue;
        }
        const long base = (((long)n * g.Co + k) * g.Ho + ho) * g.Wo + wo;
        Elem<bf16>::store(p.out, base, y0);
        if (w1) Elem<bf16>::store(p.out, base + 1, y1);
    }
}

static int fused_ci_pad(const WinoGeom &g) { return (g.Ci + kFuC - 1) / kFuC * kFuC; }

size_t winograd_fused_ws_bytes(const Dims &d, int op)
{
    const WinoGeom g = geom(d, op, 1, 2);
    return (size_t)64 * fused_ci_pad(g) * g.Mo4;
}

template <class E>
static hipError_t winograd_fused_run(const Dims &d, int op, int b, const void *in, const void *w, void *out,
                                     float *ws, bool filter_ready, hipStream_t s)
{
    const WinoGeom g = geom(d, op, b, 2);
    const bool phased = g.sh * g.sw > 1;
    LaunchLog *log = launch_log();
    // bf16 tensors: the kernel on the bf16 matrix pipe (UCD_FUSED_BF16_FP32=1 in the environment keeps the
    // fp32 products, for comparison); images of fewer than 4 pixels would break its address arithmetic
    static const bool bf16_fp32 = getenv("UCD_FUSED_BF16_FP32") != nullptr;
    const bool bf16_pipe = std::is_same_v<E, bf16> && !bf16_fp32 && g.Hi * g.Wi >= 4;
    const int ci_pad16 = (g.Ci + kBfC - 1) / kBfC * kBfC;
    if (filter_ready) {
        // U of this filter is still in the workspace from the previous micro-batch
    } else if (log) log->add(phased ? "wino_phase_filter_kernel" : bf16_pipe ? "wino_filter_bf16_kernel" : "wino_filter_kernel");
    else if (bf16_pipe && phased)
        wino_phase_filter_bf16_kernel<E><<<(unsigned)((ci_pad16 * g.Mo4 + 255) / 256), 256, 0, s>>>(
            w, (uint16_t *)ws, d.K, d.C, d.R, d.S, d.sh, d.sw, g.Mo4, ci_pad16);
    else if (bf16_pipe)
        wino_filter_bf16_kernel<E><<<(unsigned)((ci_pad16 * g.Mo4 + 255) / 256), 256, 0, s>>>(
            w, (uint16_t *)ws, g.Ci, g.Co, g.Mo4, g.transposed ? 1 : 0, ci_pad16);
    else if (phased)
        wino_phase_filter_kernel<E><<<(unsigned)((fused_ci_pad(g) * g.Mo4 + 255) / 256), 256, 0, s>>>(
            w, ws, d.K, d.C, d.R, d.S, d.sh, d.sw, g.Mo4, fused_ci_pad(g));
    else
        wino_filter_kernel<E, 2><<<(unsigned)((fused_ci_pad(g) * g.Mo4 + 255) / 256), 256, 0, s>>>(
            w, ws, g.Ci, g.Co, g.Mo4, g.transposed ? 1 : 0, fused_ci_pad(g));
    hipError_t e = log ? hipSuccess : hipGetLastError();
    if (e != hipSuccess) return e;
    if (bf16_pipe) {
        const int ci_pad = ci_pad16;
        FusedBf16Params q{};
        q.lead = (int)(((uintptr_t)in >> 1) & 1);
        q.in = (const char *)in - 2 * q.lead; q.U = ws; q.out = out;
        q.in_bytes = (uint32_t)((2 * (size_t)q.lead + 2 * (size_t)b * g.Ci * g.Hi * g.Wi + 3) / 4 * 4);
        q.ci_pad = ci_pad;
        q.u_bytes = (uint32_t)((size_t)32 * ci_pad * g.Mo4);
        q.g = g; q.divT = FastDiv(g.T); q.divTW = FastDiv(g.TW);
        q.n_tiles = b * g.T;
        q.k_blocks = (g.Co + kFuK - 1) / kFuK;
        const unsigned nb = (unsigned)(q.k_blocks * ((q.n_tiles + kFuT - 1) / kFuT));
        if (log) {
            log->add(std::string(phased ? "wino_fused_bf16_kernel<phases>" : "wino_fused_bf16_kernel") + " blocks=" + std::to_string(nb) + " gemm_flops=" +
                     std::to_string(2.0 * 16 * g.Co * (double)q.n_tiles * g.Ci));
            return hipSuccess;
        }
        if (phased) wino_fused_bf16_kernel<true><<<nb, 512, 0, s>>>(q);
        else wino_fused_bf16_kernel<false><<<nb, 512, 0, s>>>(q);
        return hipGetLastError();
    }
    FusedParams p{};
    p.in = in; p.U = ws; p.out = out;
    p.in_bytes = (uint32_t)(Elem<E>::kBytes * (size_t)b * g.Ci * g.Hi * g.Wi);
    p.ci_pad = fused_ci_pad(g);
    p.u_bytes = (uint32_t)((size_t)64 * p.ci_pad * g.Mo4);
    p.g = g; p.divT = FastDiv(g.T); p.divTW = FastDiv(g.TW);
    p.n_tiles = b * g.T;
    // row-vector patch loads: fp32 tensors (UCD_FUSED_ELEMENTWISE=1 in the environment keeps the
    // element-wise loads, for comparison).  With them, the 128 x 32 block wherever 128-channel blocks
    // cover the output channels with no more padding than 64-channel ones (UCD_FUSED_NARROW=1: never).
    static const bool elementwise = getenv("UCD_FUSED_ELEMENTWISE") != nullptr;
    static const bool narrow = getenv("UCD_FUSED_NARROW") != nullptr;
    const bool rows = std::is_same_v<E, float> && !elementwise && g.pad_w <= 2;
    const bool wide = rows && !phased && !narrow && (g.Co + 127) / 128 * 2 <= (g.Co + 63) / 64;
    const int kblock = wide ? 128 : kFuK, tblock = wide ? 32 : kFuT;
    p.k_blocks = (g.Co + kblock - 1) / kblock;
    const unsigned blocks = (unsigned)(p.k_blocks * ((p.n_tiles + tblock - 1) / tblock));
    if (log) {
        log->add(std::string(phased ? "wino_fused_kernel<phases>" : "wino_fused_kernel") + " blocks=" +
                 std::to_string(blocks) + " gemm_flops=" + std::to_string(2.0 * 16 * g.Co * (double)p.n_tiles * g.Ci));
        return hipSuccess;
    }
    if (phased) {
        if (rows) wino_fused_kernel<float, 2, false, true><<<blocks, 256, 0, s>>>(p);
        else wino_fused_kernel<E, -1, false, true><<<blocks, 256, 0, s>>>(p);
        return hipGetLastError();
    }
    if constexpr (std::is_same_v<E, float>) {
        const bool odd = g.Wi % 2 != 0;
        if (wide) {
            if (g.pad_w == 0) wino_fused_kernel<E, 0, false, false, true><<<blocks, 256, 0, s>>>(p);
            else if (g.pad_w == 2) wino_fused_kernel<E, 2, false, false, true><<<blocks, 256, 0, s>>>(p);
            else if (odd) wino_fused_kernel<E, 1, true, false, true><<<blocks, 256, 0, s>>>(p);
            else wino_fused_kernel<E, 1, false, false, true><<<blocks, 256, 0, s>>>(p);
        } else if (rows) {
            if (g.pad_w == 0) wino_fused_kernel<E, 0><<<blocks, 256, 0, s>>>(p);
            else if (g.pad_w == 2) wino_fused_kernel<E, 2><<<blocks, 256, 0, s>>>(p);
            else if (odd) wino_fused_kernel<E, 1, true><<<blocks, 256, 0, s>>>(p);
            else wino_fused_kernel<E, 1, false><<<blocks, 256, 0, s>>>(p);
        }
    }
    if (!rows) wino_fused_kernel<E, -1><<<blocks, 256, 0, s>>>(p);
    return hipGetLastError();
}

hipError_t winograd_fused(const Dims &d, int op, int b, const void *in, const void *w, void *out, float *ws,
                          bool filter_ready, hipStream_t s)
{
    return d.dtype == 1 ? winograd_fused_run<bf16>(d, op, b, in, w, out, ws, filter_ready, s)
                        : winograd_fused_run<float>(d, op, b, in, w, out, ws, filter_ready, s);
}

// D[xi][k][j] = (A dy A^T)[xi] for the m x m tile j of dy (zero outside the image), lanes along j.
// g is the Forward geometry: Co = K, Ho x Wo = P x Q.
template <class E, int MT>
__global__ __launch_bounds__(256) void wino_grad_kernel(const void *__restrict__ dy, float *__restrict__ D,
                                                        WinoGeom g, FastDiv divT, FastDiv divTW, int n_tiles)
{
    constexpr int A = Wino<MT>::A;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= g.ld) return;
    const size_t plane = (size_t)g.Co * g.ld;
    uint32_t n = 0, t, th = 0, tw = 0;
    if (j < n_tiles) {
        divT.divmod((uint32_t)j, n, t);
        divTW.divmod(t, th, tw);
    }
    const int h0 = MT * (int)th, w0 = MT * (int)tw;
    for (int co = blockIdx.y; co < g.Co; co += gridDim.y) {
        const size_t src = ((size_t)n * g.Co + co) * g.Ho * g.Wo;
        float tr[A][MT];  // A dy, column by column
#pragma unroll
        for (int s = 0; s < MT; ++s) {
            float z[MT], u[A];
#pragma unroll
            for (int r = 0; r < MT; ++r)
                z[r] = (j < n_tiles && h0 + r < g.Ho && w0 + s < g.Wo) ? Elem<E>::get(dy, src + (h0 + r) * g.Wo + w0 + s)
                                                                      : 0.f;
            Wino<MT>::grad(z, u);
#pragma unroll
            for (int r = 0; r < A; ++r) tr[r][s] = u[r];
        }
        float *dst = D + (size_t)co * g.ld + j;
#pragma unroll
        for (int r = 0; r < A; ++r) {
            float u[A];
            Wino<MT>::grad(tr[r], u);
#pragma unroll
            for (int s = 0; s < A; ++s) dst[(size_t)(r * A + s) * plane] = u[s];
        }
    }
}

// dw[k, c] = beta * dw[k, c] + G^T Mw[., k, c] G, one thread per (k, c)
template <int MT>
__global__ __launch_bounds__(256) void wino_dw_kernel(const float *__restrict__ Mw, float *__restrict__ dw, int KC,
                                                      float beta)
{
    constexpr int A = Wino<MT>::A;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= KC) return;
    float tr[3][A];  // G^T Mw, column by column
#pragma unroll
    for (int s = 0; s < A; ++s) {
        float m[A], w3[3];
#pragma unroll
        for (int r = 0; r < A; ++r) m[r] = Mw[(size_t)(r * A + s) * KC + i];
        Wino<MT>::filter_t(m, w3);
#pragma unroll
        for (int r = 0; r < 3; ++r) tr[r][s] = w3[r];
    }
    float *dst = dw + (size_t)i * 9;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        float w3[3];
        Wino<MT>::filter_t(tr[r], w3);
#pragma unroll
        for (int s = 0; s < 3; ++s) dst[r * 3 + s] = beta == 0.f ? w3[s] : beta * dst[r * 3 + s] + w3[s];
    }
}

// ---- BackwardFilter F(3x3,2x2) with both data transforms fused into the GEMM kernel -------------------
// Mw[xi][k][c] = sum over tiles of D[xi][k][tile] * V[xi][c][tile] with D = A dy A^T and V = B^T x B
// computed on the fly; the workspace holds Mw alone (64*K*C bytes).  A workgroup owns 64 output
// channels x 64 input channels for all 16 points (16 accumulator tiles per wave, as in the kernel
// above) and reduces over a chunk of the tiles: 8 tile positions of the image (fixed for the
// workgroup, so that every thread's patch addresses and border masks are computed once) times a range
// of images, one image per step.  Per step a thread fetches and transforms the x patches of two
// (input channel, tile) pairs and the dy tiles of two (output channel, tile) pairs; 64 MFMAs per
// wave (16 points x 4 tile pairs).  Chunks meet in Mw through fp32 atomics; dw = beta*dw + G^T Mw G
// is wino_dw_kernel's.
constexpr int kFwT = 8;                 // tile positions per step (the MFMAs' reduction rows)
constexpr int kFwLd = 64;               // LDS row stride; column c of tile position t sits at c ^ 4t (see kernel)
constexpr int kFwPairs = kFwT / 2;

struct FusedFilterParams {
    const void *x, *dy;
    float *Mw;
    uint32_t x_bytes, dy_bytes;
    WinoGeom g;       // Forward geometry: Ci = C, Co = K, Hi x Wi = H x W, Ho x Wo = P x Q
    int b, k_blocks, c_blocks, groups, n_split, images_per_chunk;
    // The last tile-position group when the image leaves it 1, 2 or 4 tiles (49 tiles: 1): instead of
    // padding it to 8 positions, its 8 slots are those tiles of `spread` = 8, 4 or 2 consecutive images,
    // and it takes `spread` images per step.  1: off.  The workgroups of that group come after all others
    // and take the whole micro-batch each (b / spread steps: shorter than a chunk of the others).
    int spread;
};

// PW >= 0 (fp32 tensors, horizontal padding PW = 0 or 1): patch rows of x and tile rows of dy are
// fetched as 8-, 12- or 16-byte windows instead of element by element, as in wino_fused_kernel (the
// element loads keep the texture path at 0.87 cache accesses per cycle, i.e. saturated): the window
// of x starts at column 2*tw; with PW = 1 the patch's first column comes from the lane below (the
// tile to the left, same channel), except for the first tile position of a group, which fetches it.
template <class E, int PW, bool ODD_W = false>
__global__ __launch_bounds__(256) void wino_fused_filter_kernel(FusedFilterParams p)
{
    constexpr uint32_t EB = Elem<E>::kBytes;
    constexpr bool kRows = PW >= 0;
    static_assert(!kRows || EB == 4, "row loads are written for fp32 tensors");
    __shared__ __attribute__((aligned(16))) float Ds[2][16][kFwT][kFwLd];
    __shared__ __attribute__((aligned(16))) float Vs[2][16][kFwT][kFwLd];
    const WinoGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int wk = wave & 1, wc = wave >> 1;

    // work item: (output-channel block, input-channel block, tile-position group, image chunk);
    // neighbours on an XCD share the x patches (same input-channel block, group and chunk)
    uint32_t v = xcd_order(blockIdx.x, gridDim.x);
    const int kb = (int)(v % (uint32_t)p.k_blocks); v /= (uint32_t)p.k_blocks;
    const int cb = (int)(v % (uint32_t)p.c_blocks); v /= (uint32_t)p.c_blocks;
    // chunked groups first (group fastest, then chunk), then the spread group's whole-batch workgroups
    const int chunked = p.groups - (p.spread > 1 ? 1 : 0);
    const bool whole = (int)v >= chunked * p.n_split;
    const int grp = whole ? p.groups - 1 : (int)(v % (uint32_t)chunked);
    const int chunk = whole ? 0 : (int)(v / (uint32_t)chunked);
    const int k0 = kb * 64, c0 = cb * 64;
    const int n_begin = whole ? 0 : chunk * p.images_per_chunk, n_end = whole ? p.b : min(p.b, n_begin + p.images_per_chunk);
    // images per step: 1, or for the last group `spread` (slot s = tile s % L of image s / L, L = 8 / spread;
    // slots of images past the batch read out of range, i.e. zeros)
    const int n_step = whole ? p.spread : 1;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc_bytes(p.x, 0, p.x_bytes);
    const __amdgpu_buffer_rsrc_t rdy = make_rsrc_bytes(p.dy, 0, p.dy_bytes);

    // producer role: tile position tid % 8 of the group, channel tid / 8 (and + 32) of both blocks;
    // offsets within image 0 (kOob: outside the image, or no such tile / channel).
    // LDS slabs are [point][tile position][64 channels] with channel c of tile position t stored at
    // column c ^ 4t: a wave's store (8 tile positions x 8 channels) then covers all banks evenly, and
    // with a row stride of 64 every operand read is one base register (per tile pair) plus an
    // immediate offset.
    const int ptile = tid & 7, pch = tid >> 3;
    const int pcol = pch ^ (4 * ptile);   // + 32 h: bit 5 is not touched by the swizzle
    // element-wise: vx = the 16 pixels of the patch, vd = the 4 of the dy tile.  Rows: vx[h][r] = the
    // window start of patch row r, vx[h][4 + r] = its first column where this lane fetches it itself;
    // vd[h][r] = the start of tile row r.
    uint32_t vx[2][kRows ? 8 : 16], vd[2][kRows ? 2 : 4];
    bool own_col = false, ok1 = true, ok2 = true, ok3 = true, dy_ok1 = true;
    {
        const int per_image = kFwT / n_step;   // slots per image
        const int t = grp * kFwT + ptile % per_image, image = ptile / per_image;
        const bool live = t < g.T;
        const int th = live ? t / g.TW : 0, tw = live ? t % g.TW : 0;
        const int h0 = 2 * th - g.pad_h, w0 = 2 * tw - g.pad_w;
        const uint32_t x_slot = EB * (uint32_t)(image * g.Ci * g.Hi * g.Wi), dy_slot = EB * (uint32_t)(image * g.Co * g.Ho * g.Wo);
        if constexpr (kRows) {
            const int ws = 2 * tw;   // = w0 + PW
            // the first column is this lane's own load (or the padding's 0) for the first tile position
            // of a group (of each image's share of it) and for tiles in the first tile column; otherwise
            // the lane below holds it
            own_col = ptile % per_image == 0 || tw == 0;
            ok1 = ws + 1 < g.Wi; ok2 = ws + 2 < g.Wi; ok3 = ws + 3 < g.Wi;
            dy_ok1 = 2 * tw + 1 < g.Wo;
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int c = c0 + pch + 32 * h, k = k0 + pch + 32 * h;
            if constexpr (kRows) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int hh = h0 + r;
                    const bool ok = live && c < g.Ci && (unsigned)hh < (unsigned)g.Hi;
                    const uint32_t row = EB * (uint32_t)((c * g.Hi + hh) * g.Wi + 2 * tw) + x_slot;
                    vx[h][r] = ok ? row : kOob;
                    vx[h][4 + r] = ok && PW == 1 && ptile % per_image == 0 && tw > 0 ? row - EB : kOob;
                }
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const int hh = 2 * th + r;
                    const bool ok = live && k < g.Co && hh < g.Ho;
                    vd[h][r] = ok ? EB * (uint32_t)((k * g.Ho + hh) * g.Wo + 2 * tw) + dy_slot : kOob;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int hh = h0 + r, ww = w0 + q;
                        const bool ok = live && c < g.Ci && (unsigned)hh < (unsigned)g.Hi && (unsigned)ww < (unsigned)g.Wi;
                        vx[h][4 * r + q] = ok ? EB * (uint32_t)((c * g.Hi + hh) * g.Wi + ww) + x_slot : kOob;
                    }
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const int hh = 2 * th + r, ww = 2 * tw + q;
                        const bool ok = live && k < g.Co && hh < g.Ho && ww < g.Wo;
                        vd[h][2 * r + q] = ok ? EB * (uint32_t)((k * g.Ho + hh) * g.Wo + ww) + dy_slot : kOob;
                    }
            }
        }
    }
    const uint32_t x_image = EB * (uint32_t)(g.Ci * g.Hi * g.Wi), dy_image = EB * (uint32_t)(g.Co * g.Ho * g.Wo);

    float dx[2][16], dz[2][4];  // the thread's patches of the image after the one in LDS
    float dl[2][4];             // rows, PW = 1: the first column where the lane fetches it itself
    constexpr int kXLoads = !kRows ? 16 : PW == 1 ? 8 : 4, kDyLoads = kRows ? 2 : 4;   // load instructions per patch / tile
    // an image past the chunk's end gets a scalar offset that pushes every address out of range
    auto fetch_x = [&](int n, int h, int i) {   // i < kXLoads
        const uint32_t so = n < n_end ? (uint32_t)n * x_image : kOob;
        if constexpr (!kRows) {
            dx[h][i] = Elem<E>::load(rx, vx[h][i], so);
        } else if constexpr (PW == 0) {
            const f32x4 q = buf_load4(rx, vx[h][i], so);
            dx[h][4 * i] = q.x; dx[h][4 * i + 1] = q.y; dx[h][4 * i + 2] = q.z; dx[h][4 * i + 3] = q.w;
        } else if (i < 4) {
            const auto q = __builtin_amdgcn_raw_buffer_load_b96(rx, (int)vx[h][i], (int)so, 0);
#pragma unroll
            for (int c = 0; c < 3; ++c) dx[h][4 * i + 1 + c] = __uint_as_float(q[c]);
        } else {
            dl[h][i - 4] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rx, (int)vx[h][i], (int)so, 0));
        }
    };
    auto fetch_dy = [&](int n, int h, int i) {   // i < kDyLoads
        const uint32_t so = n < n_end ? (uint32_t)n * dy_image : kOob;
        if constexpr (!kRows) {
            dz[h][i] = Elem<E>::load(rdy, vd[h][i], so);
        } else {
            const auto q = __builtin_amdgcn_raw_buffer_load_b64(rdy, (int)vd[h][i], (int)so, 0);
            dz[h][2 * i] = __uint_as_float(q[0]);
            dz[h][2 * i + 1] = __uint_as_float(q[1]);
        }
    };
    // rows: the windows as loaded become the patch / tile (see wino_fused_kernel)
    auto finish_x = [&](int h) {
        if constexpr (kRows) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (PW == 1) {
                    if constexpr (ODD_W) dx[h][4 * r + 2] = ok1 ? dx[h][4 * r + 2] : 0.f;
                    dx[h][4 * r + 3] = ok2 ? dx[h][4 * r + 3] : 0.f;
                    const int left = __builtin_amdgcn_update_dpp(0, (int)__float_as_uint(dx[h][4 * r + 2]), 0x138, 0xf, 0xf, false);
                    dx[h][4 * r] = own_col ? dl[h][r] : __uint_as_float((uint32_t)left);
                } else {
                    if constexpr (ODD_W) dx[h][4 * r + 3] = ok3 ? dx[h][4 * r + 3] : 0.f;
                }
            }
        }
    };
    auto finish_dy = [&](int h) {
        if constexpr (kRows && ODD_W) {   // an odd width of x is an odd width of dy (3x3, stride 1, equal padding)
            dz[h][1] = dy_ok1 ? dz[h][1] : 0.f;
            dz[h][3] = dy_ok1 ? dz[h][3] : 0.f;
        }
    };
    auto store_v = [&](int buf, int h) {  // B^T x B of patch h
        finish_x(h);
        float tr[16];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float a0 = dx[h][c], a1 = dx[h][4 + c], a2 = dx[h][8 + c], a3 = dx[h][12 + c];
            tr[c] = a0 - a2;
            tr[4 + c] = a1 + a2;
            tr[8 + c] = a2 - a1;
            tr[12 + c] = a1 - a3;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float a0 = tr[4 * r], a1 = tr[4 * r + 1], a2 = tr[4 * r + 2], a3 = tr[4 * r + 3];
            Vs[buf][4 * r + 0][ptile][pcol + 32 * h] = a0 - a2;
            Vs[buf][4 * r + 1][ptile][pcol + 32 * h] = a1 + a2;
            Vs[buf][4 * r + 2][ptile][pcol + 32 * h] = a2 - a1;
            Vs[buf][4 * r + 3][ptile][pcol + 32 * h] = a1 - a3;
        }
    };
    auto store_d = [&](int buf, int h) {  // A dy A^T of tile h: rows (z0, z0+z1, z0-z1, -z1) of A z, then the same on columns
        finish_dy(h);
        const float z00 = dz[h][0], z01 = dz[h][1], z10 = dz[h][2], z11 = dz[h][3];
        const float t[4][2] = {{z00, z01}, {z00 + z10, z01 + z11}, {z00 - z10, z01 - z11}, {-z10, -z11}};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            Ds[buf][4 * r + 0][ptile][pcol + 32 * h] = t[r][0];
            Ds[buf][4 * r + 1][ptile][pcol + 32 * h] = t[r][0] + t[r][1];
            Ds[buf][4 * r + 2][ptile][pcol + 32 * h] = t[r][0] - t[r][1];
            Ds[buf][4 * r + 3][ptile][pcol + 32 * h] = -t[r][1];
        }
    };

    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < kXLoads; ++i) fetch_x(n_begin, h, i);
#pragma unroll
        for (int i = 0; i < kDyLoads; ++i) fetch_dy(n_begin, h, i);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        store_v(0, h);
        store_d(0, h);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < kXLoads; ++i) fetch_x(n_begin + n_step, h, i);
#pragma unroll
        for (int i = 0; i < kDyLoads; ++i) fetch_dy(n_begin + n_step, h, i);
    }
    __syncthreads();

    int col_q[kFwPairs];   // the lane's column within its wave's 32, as stored for tile position 2q + lhi
#pragma unroll
    for (int q = 0; q < kFwPairs; ++q) col_q[q] = l32 ^ (4 * (2 * q + lhi));

    int buf = 0;
    for (int n = n_begin; n < n_end; n += n_step) {
        // operands of (point xi, tile pair q): rows 2q + lhi of the point's slab (columns swizzled by
        // 4 (2q + lhi)), read one point ahead
        const float *da = &Ds[buf][0][lhi][wk * 32];
        const float *vb = &Vs[buf][0][lhi][wc * 32];
        float a[2][kFwPairs], b[2][kFwPairs];
        auto read_ops = [&](int xi) {
#pragma unroll
            for (int q = 0; q < kFwPairs; ++q) {
                a[xi & 1][q] = da[(xi * kFwT + 2 * q) * kFwLd + col_q[q]];
                b[xi & 1][q] = vb[(xi * kFwT + 2 * q) * kFwLd + col_q[q]];
            }
        };
        read_ops(0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(UCD_MFMA_PRIO);
        auto slot = [&](auto M) {
            constexpr int m = decltype(M)::value;
            constexpr int xi = m / kFwPairs, q = m % kFwPairs;
            acc[xi] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[xi & 1][q], b[xi & 1][q], acc[xi], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (q == 0 && xi + 1 < 16) read_ops(xi + 1);
            // image n + 1 (in registers) is transformed into the other LDS buffer and every register
            // reloaded with image n + 2 as soon as it is free: one piece, and at most one global load,
            // behind each MFMA (a burst of loads would block this SIMD's only wave)
            constexpr int kXSlots = 1 + kXLoads, kDySlots = 1 + kDyLoads, kDyStart = 1 + 2 * kXSlots;
            if constexpr (m >= 1 && m < kDyStart) {                      // x patches: 2 x (transform + loads)
                constexpr int h = (m - 1) / kXSlots, i = (m - 1) % kXSlots;
                if constexpr (i == 0) store_v(buf ^ 1, h);
                else fetch_x(n + 2 * n_step, h, i - 1);
            }
            if constexpr (m >= kDyStart && m < kDyStart + 2 * kDySlots) {  // dy tiles: 2 x (transform + loads)
                constexpr int h = (m - kDyStart) / kDySlots, i = (m - kDyStart) % kDySlots;
                if constexpr (i == 0) store_d(buf ^ 1, h);
                else fetch_dy(n + 2 * n_step, h, i - 1);
            }
            static_assert(kDyStart + 2 * kDySlots <= 16 * kFwPairs, "the step's work fits behind its MFMAs");
            __builtin_amdgcn_sched_barrier(0);
        };
        static_for<16 * kFwPairs>(slot);
        __builtin_amdgcn_s_setprio(0);
        __syncthreads();
        buf ^= 1;
    }

    // lane = input channel (column l32 of the wave's 32), register e = output-channel row
    const int c = c0 + wc * 32 + l32;
    if (c >= g.Ci) return;
    const size_t plane = (size_t)g.Co * g.Ci;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int k = k0 + wk * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
        if (k >= g.Co) continue;
#pragma unroll
        for (int xi = 0; xi < 16; ++xi) unsafeAtomicAdd(p.Mw + xi * plane + (size_t)k * g.Ci + c, acc[xi][e]);
    }
}

size_t winograd_fused_filter_ws_bytes(const Dims &d) { return (size_t)64 * d.K * d.C; }

template <class E>
static hipError_t winograd_fused_filter_run(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                                            float *ws, hipStream_t s)
{
    const WinoGeom g = geom(d, 0, b, 2);
    const int KC = d.K * d.C;
    hipError_t e = fill_zero(ws, (size_t)16 * KC, s);
    if (e != hipSuccess) return e;
    FusedFilterParams p{};
    p.x = x; p.dy = dy; p.Mw = ws;
    p.x_bytes = xbytes(d, b); p.dy_bytes = ybytes(d, b);
    p.g = g; p.b = b;
    p.k_blocks = (d.K + 63) / 64; p.c_blocks = (d.C + 63) / 64; p.groups = (g.T + kFwT - 1) / kFwT;
    const int left = g.T % kFwT;   // tiles in the last group
    p.spread = b >= 8 && (left == 1 || left == 2 || left == 4) ? kFwT / left : 1;
    // image chunks (of all groups but a spread one).  A workgroup costs its steps plus about 11 steps' worth
    // of start-up and of adding its 16 accumulator tiles into Mw (measured on 13x13 layers at two chunk
    // sizes); the launch costs the rounds of one workgroup per CU times that.  The chunk count with the
    // lowest such cost, chunks of at least 4 images.
    const long per_group = (long)p.k_blocks * p.c_blocks, cus = device_cus();
    const long items = per_group * (p.groups - (p.spread > 1 ? 1 : 0));
    long split = 1;
    if (items > 0) {
        const long cap = b / 4 < 1 ? 1 : b / 4;
        double best = 1e30;
        for (long c = 1; c <= cap && c <= 64; ++c) {
            const int per = (int)((b + c - 1) / c);
            const long wgs = items * ((b + per - 1) / per) + (p.spread > 1 ? per_group : 0);
            const double cost = (double)((wgs + cus - 1) / cus) * (per + 11.0);
            if (cost < best - 1e-9) { best = cost; split = c; }
        }
    }
    p.images_per_chunk = (int)((b + split - 1) / split);
    p.n_split = (b + p.images_per_chunk - 1) / p.images_per_chunk;
    const unsigned blocks = (unsigned)(items * p.n_split + (p.spread > 1 ? per_group : 0));
    LaunchLog *log = launch_log();
    if (log) {
        // tile slots multiplied per image: whole groups of 8, the last one shared by `spread` images
        const double slots = p.spread > 1 ? (double)(p.groups - 1) * kFwT + (double)kFwT / p.spread : (double)p.groups * kFwT;
        log->add("wino_fused_filter_kernel blocks=" + std::to_string(blocks) + " gemm_flops=" +
                 std::to_string(2.0 * 16 * d.K * (double)d.C * slots * b));
        log->add("wino_dw_kernel");
        return hipSuccess;
    }
    // row-vector loads: fp32 tensors, horizontal padding 0 or 1 (UCD_FUSED_ELEMENTWISE=1 keeps the
    // element-wise loads, for comparison)
    static const bool elementwise = getenv("UCD_FUSED_ELEMENTWISE") != nullptr;
    bool rows = false;
    if constexpr (std::is_same_v<E, float>) {
        rows = !elementwise && (g.pad_w == 0 || g.pad_w == 1);
        const bool odd = g.Wi % 2 != 0;
        if (rows && g.pad_w == 0 && odd) wino_fused_filter_kernel<E, 0, true><<<blocks, 256, 0, s>>>(p);
        else if (rows && g.pad_w == 0) wino_fused_filter_kernel<E, 0, false><<<blocks, 256, 0, s>>>(p);
        else if (rows && odd) wino_fused_filter_kernel<E, 1, true><<<blocks, 256, 0, s>>>(p);
        else if (rows) wino_fused_filter_kernel<E, 1, false><<<blocks, 256, 0, s>>>(p);
    }
    if (!rows) wino_fused_filter_kernel<E, -1><<<blocks, 256, 0, s>>>(p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    wino_dw_kernel<2><<<(unsigned)((KC + 255) / 256), 256, 0, s>>>(ws, dw, KC, beta);
    return hipGetLastError();
}

hipError_t winograd_fused_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                                 float *ws, hipStream_t s)
{
    return d.dtype == 1 ? winograd_fused_filter_run<bf16>(d, b, x, dy, dw, beta, ws, s)
                        : winograd_fused_filter_run<float>(d, b, x, dy, dw, beta, ws, s);
}

template <class E, int MT>
static hipError_t winograd_filter_run(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                                      float *ws, hipStream_t s)
{
    constexpr int AA = Wino<MT>::A * Wino<MT>::A;
    const WinoGeom g = geom(d, 0, b, MT);
    const int n_tiles = b * g.T, KC = d.K * d.C;
    float *Mw = ws;
    float *V = Mw + (size_t)AA * KC;
    float *D = V + (size_t)AA * d.C * g.ld;
    const FastDiv divT(g.T), divTW(g.TW);

    LaunchLog *log = launch_log();
    hipError_t e = fill_zero(Mw, (size_t)AA * KC, s);
    if (e != hipSuccess) return e;
    dim3 gi((unsigned)((g.ld + 255) / 256), (unsigned)(d.C < 4096 ? d.C : 4096));
    dim3 gd((unsigned)((g.ld + 255) / 256), (unsigned)(d.K < 4096 ? d.K : 4096));
    if (log) {
        log->add("wino_input_kernel");
        log->add("wino_grad_kernel");
    } else {
        wino_input_kernel<E, MT><<<gi, 256, 0, s>>>(x, V, g, divT, divTW, n_tiles);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        wino_grad_kernel<E, MT><<<gd, 256, 0, s>>>(dy, D, g, divT, divTW, n_tiles);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }

    GemmShape gs{d.K, d.C, n_tiles};
    gs.batch = AA;
    gs.a_batch = (long)d.K * g.ld;
    gs.b_batch = (long)d.C * g.ld;
    gs.c_batch = KC;
    gs.splits = filter_splits(gs.M, gs.N, gs.Kd, AA);
    KLaneParams pa{};
    pa.t = D; pa.bytes = (uint32_t)(gs.a_batch * 4); pa.row_stride = 1; pa.col_stride = g.ld;
    KLaneParams pb{};
    pb.t = V; pb.bytes = (uint32_t)(gs.b_batch * 4); pb.row_stride = 1; pb.col_stride = g.ld;
    EpiDenseParams pe{Mw, d.C};
    if ((e = launch_gemm<KLane0, KLane0, EpiAtomic, true>(pa, pb, pe, gs, s)) != hipSuccess) return e;

    if (log) {
        log->add("wino_dw_kernel");
        return hipSuccess;
    }
    wino_dw_kernel<MT><<<(unsigned)((KC + 255) / 256), 256, 0, s>>>(Mw, dw, KC, beta);
    return hipGetLastError();
}

hipError_t winograd_bwd_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta,
                               float *ws, int mt, hipStream_t s)
{
    const bool h = d.dtype == 1;
    if (mt == 2)
        return h ? winograd_filter_run<bf16, 2>(d, b, x, dy, dw, beta, ws, s)
                 : winograd_filter_run<float, 2>(d, b, x, dy, dw, beta, ws, s);
    if (mt == 4)
        return h ? winograd_filter_run<bf16, 4>(d, b, x, dy, dw, beta, ws, s)
                 : winograd_filter_run<float, 4>(d, b, x, dy, dw, beta, ws, s);
    return hipErrorInvalidValue;
}

template <class E>
static hipError_t winograd_any(const Dims &d, int op, int b, const void *in, const void *w, void *out, float *ws,
                               bool filter_ready, int mt, hipStream_t s)
{
    if (mt == 2) return winograd_run<E, 2>(d, op, b, in, w, out, ws, filter_ready, s);
    if (mt == 4) return winograd_run<E, 4>(d, op, b, in, w, out, ws, filter_ready, s);
    return hipErrorInvalidValue;
}

hipError_t winograd_fwd(const Dims &d, int b, const void *x, const void *w, void *y, float *ws, bool filter_ready,
                        int mt, hipStream_t s)
{
    return d.dtype == 1 ? winograd_any<bf16>(d, 0, b, x, w, y, ws, filter_ready, mt, s)
                        : winograd_any<float>(d, 0, b, x, w, y, ws, filter_ready, mt, s);
}

hipError_t winograd_bwd_data(const Dims &d, int b, const void *dy, const void *w, void *dx, float *ws,
                             bool filter_ready, int mt, hipStream_t s)
{
    return d.dtype == 1 ? winograd_any<bf16>(d, 1, b, dy, w, dx, ws, filter_ready, mt, s)
                        : winograd_any<float>(d, 1, b, dy, w, dx, ws, filter_ready, mt, s);
}

}  // namespace ucd
