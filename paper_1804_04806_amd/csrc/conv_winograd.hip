// Winograd F(2x2,3x3) convolution (Lavin & Gray) for 3x3 stride-1 layers, Forward and
// BackwardData, with every transform buffer in the caller's workspace:
//   U[16][Ci][Mo4]   filter transform  U = G g G^T            (Mo4 = out channels rounded up to 4)
//   V[16][Ci][ld]    input transform   V = B^T d B  per 4x4 input tile at stride 2
//   Z[16][Mo][ld]    16 independent GEMMs  Z_xi = U_xi^T[Mo x Ci] * V_xi[Ci x b*T]   (MFMA)
//   out              output transform  y = A^T z A  per 2x2 output tile
// with T = ceil(Ho/2) * ceil(Wo/2) tiles per image and ld = b*T rounded up to 4.
// BackwardData is the same pipeline on dy with the filter's two channel indices swapped and its
// taps reversed, and padding 2 - pad.
#include "gemm_launch.hpp"
#include "kernels.h"

namespace ucd {

struct WinoGeom {
    int Ci, Co, Hi, Wi, Ho, Wo, pad_h, pad_w;
    int TH, TW, T;
    int Mo4, ld;
    bool transposed;  // BackwardData: filter read as w[ci][co] with reversed taps
};

static WinoGeom geom(const Dims &d, int op, int b)
{
    WinoGeom g;
    if (op == 0) {
        g.Ci = d.C; g.Co = d.K; g.Hi = d.H; g.Wi = d.W; g.Ho = d.P; g.Wo = d.Q;
        g.pad_h = d.ph; g.pad_w = d.pw; g.transposed = false;
    } else {
        g.Ci = d.K; g.Co = d.C; g.Hi = d.P; g.Wi = d.Q; g.Ho = d.H; g.Wo = d.W;
        g.pad_h = 2 - d.ph; g.pad_w = 2 - d.pw; g.transposed = true;
    }
    g.TH = (g.Ho + 1) / 2; g.TW = (g.Wo + 1) / 2; g.T = g.TH * g.TW;
    g.Mo4 = (g.Co + 3) / 4 * 4;
    g.ld = (b * g.T + 3) / 4 * 4;
    return g;
}

bool winograd_applies(const Dims &d, int op)
{
    if (op != 0 && op != 1) return false;
    if (d.R != 3 || d.S != 3 || d.sh != 1 || d.sw != 1) return false;
    return d.ph <= 2 && d.pw <= 2;
}

size_t winograd_ws_bytes(const Dims &d, int op, int b)
{
    const WinoGeom g = geom(d, op, b);
    return (size_t)64 * ((size_t)g.Ci * g.Mo4 + (size_t)g.ld * (g.Ci + g.Co));
}

// U[xi][ci][co] = (G g G^T)[xi], one thread per (ci, co) filter; pads co up to Mo4 with zeros.
template <class E>
__global__ __launch_bounds__(256) void wino_filter_kernel(const void *__restrict__ w, float *__restrict__ U, int Ci,
                                                          int Co, int Mo4, int transposed)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= Ci * Mo4) return;
    const int ci = i / Mo4, co = i - ci * Mo4;
    float g[3][3];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            float v = 0.f;
            if (co < Co)
                v = transposed ? Elem<E>::get(w, ((size_t)(ci * Co + co) * 3 + (2 - r)) * 3 + (2 - s))
                               : Elem<E>::get(w, ((size_t)(co * Ci + ci) * 3 + r) * 3 + s);
            g[r][s] = v;
        }
    float t[4][3];  // G g
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        t[0][s] = g[0][s];
        t[1][s] = 0.5f * (g[0][s] + g[1][s] + g[2][s]);
        t[2][s] = 0.5f * (g[0][s] - g[1][s] + g[2][s]);
        t[3][s] = g[2][s];
    }
    const size_t plane = (size_t)Ci * Mo4;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float u0 = t[r][0], u1 = 0.5f * (t[r][0] + t[r][1] + t[r][2]),
                    u2 = 0.5f * (t[r][0] - t[r][1] + t[r][2]), u3 = t[r][2];
        U[(size_t)(r * 4 + 0) * plane + i] = u0;
        U[(size_t)(r * 4 + 1) * plane + i] = u1;
        U[(size_t)(r * 4 + 2) * plane + i] = u2;
        U[(size_t)(r * 4 + 3) * plane + i] = u3;
    }
}

// V[xi][ci][j] for tile j = n*T + th*TW + tw: lanes along j (coalesced plane writes).
template <class E>
__global__ __launch_bounds__(256) void wino_input_kernel(const void *__restrict__ x, float *__restrict__ V,
                                                         WinoGeom g, FastDiv divT, FastDiv divTW, int n_tiles)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= g.ld) return;
    const size_t plane = (size_t)g.Ci * g.ld;
    for (int ci = blockIdx.y; ci < g.Ci; ci += gridDim.y) {
        float d[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int s = 0; s < 4; ++s) d[r][s] = 0.f;
        if (j < n_tiles) {
            uint32_t n, t, th, tw;
            divT.divmod((uint32_t)j, n, t);
            divTW.divmod(t, th, tw);
            const int h0 = 2 * (int)th - g.pad_h, w0 = 2 * (int)tw - g.pad_w;
            const size_t src = ((size_t)n * g.Ci + ci) * g.Hi * g.Wi;
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int h = h0 + r, ww = w0 + s;
                    if ((unsigned)h < (unsigned)g.Hi && (unsigned)ww < (unsigned)g.Wi) d[r][s] = Elem<E>::get(x, src + h * g.Wi + ww);
                }
        }
        float t[4][4];  // B^T d
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            t[0][s] = d[0][s] - d[2][s];
            t[1][s] = d[1][s] + d[2][s];
            t[2][s] = d[2][s] - d[1][s];
            t[3][s] = d[1][s] - d[3][s];
        }
        float *dst = V + (size_t)ci * g.ld + j;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            dst[(size_t)(r * 4 + 0) * plane] = t[r][0] - t[r][2];
            dst[(size_t)(r * 4 + 1) * plane] = t[r][1] + t[r][2];
            dst[(size_t)(r * 4 + 2) * plane] = t[r][2] - t[r][1];
            dst[(size_t)(r * 4 + 3) * plane] = t[r][1] - t[r][3];
        }
    }
}

// out[n, co, 2th + {0,1}, 2tw + {0,1}] = A^T z A, lanes along the tile index.
template <class E>
__global__ __launch_bounds__(256) void wino_output_kernel(const float *__restrict__ Z, void *__restrict__ out,
                                                          WinoGeom g, FastDiv divT, FastDiv divTW, int n_tiles)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n_tiles) return;
    uint32_t n, t, th, tw;
    divT.divmod((uint32_t)j, n, t);
    divTW.divmod(t, th, tw);
    const int h0 = 2 * (int)th, w0 = 2 * (int)tw;
    const size_t plane = (size_t)g.Co * g.ld;
    for (int co = blockIdx.y; co < g.Co; co += gridDim.y) {
        const float *src = Z + (size_t)co * g.ld + j;
        float z[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int s = 0; s < 4; ++s) z[r][s] = src[(size_t)(r * 4 + s) * plane];
        float t[2][4];  // A^T z
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            t[0][s] = z[0][s] + z[1][s] + z[2][s];
            t[1][s] = z[1][s] - z[2][s] - z[3][s];
        }
        const size_t dst = ((size_t)n * g.Co + co) * g.Ho * g.Wo;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int h = h0 + r;
            if (h >= g.Ho) continue;
            const float y0 = t[r][0] + t[r][1] + t[r][2], y1 = t[r][1] - t[r][2] - t[r][3];
            Elem<E>::store(out, dst + h * g.Wo + w0, y0);
            if (w0 + 1 < g.Wo) Elem<E>::store(out, dst + h * g.Wo + w0 + 1, y1);
        }
    }
}

template <class E>
static hipError_t winograd_run(const Dims &d, int op, int b, const void *in, const void *w, void *out,
                               float *ws, bool filter_ready, hipStream_t s)
{
    const WinoGeom g = geom(d, op, b);
    const int n_tiles = b * g.T;
    float *U = ws;
    float *V = U + (size_t)16 * g.Ci * g.Mo4;
    float *Z = V + (size_t)16 * g.Ci * g.ld;
    const FastDiv divT(g.T), divTW(g.TW);

    LaunchLog *log = launch_log();
    if (filter_ready) {
        // U of this filter is still at the head of the workspace from the previous micro-batch
    } else if (log) log->add("wino_filter_kernel");
    else
        wino_filter_kernel<E><<<(unsigned)((g.Ci * g.Mo4 + 255) / 256), 256, 0, s>>>(w, U, g.Ci, g.Co, g.Mo4,
                                                                                  g.transposed ? 1 : 0);
    hipError_t e = log ? hipSuccess : hipGetLastError();
    if (e != hipSuccess) return e;

    dim3 gi((unsigned)((g.ld + 255) / 256), (unsigned)(g.Ci < 4096 ? g.Ci : 4096));
    if (log) log->add("wino_input_kernel");
    else
        wino_input_kernel<E><<<gi, 256, 0, s>>>(in, V, g, divT, divTW, n_tiles);
    if (!log && (e = hipGetLastError()) != hipSuccess) return e;

    GemmShape gs{g.Co, n_tiles, g.Ci};
    gs.batch = 16;
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
    wino_output_kernel<E><<<go, 256, 0, s>>>(Z, out, g, divT, divTW, n_tiles);
    return hipGetLastError();
}

hipError_t winograd_fwd(const Dims &d, int b, const void *x, const void *w, void *y, float *ws, bool filter_ready,
                        hipStream_t s)
{
    return d.dtype == 1 ? winograd_run<bf16>(d, 0, b, x, w, y, ws, filter_ready, s)
                        : winograd_run<float>(d, 0, b, x, w, y, ws, filter_ready, s);
}

hipError_t winograd_bwd_data(const Dims &d, int b, const void *dy, const void *w, void *dx, float *ws,
                             bool filter_ready, hipStream_t s)
{
    return d.dtype == 1 ? winograd_run<bf16>(d, 1, b, dy, w, dx, ws, filter_ready, s)
                        : winograd_run<float>(d, 1, b, dy, w, dx, ws, filter_ready, s);
}

}  // namespace ucd
