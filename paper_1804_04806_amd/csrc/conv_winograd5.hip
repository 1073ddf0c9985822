// Winograd F(2x2,5x5) with the data transforms fused into the GEMM kernel: Forward and BackwardData
// of 5x5 stride-1 layers with horizontal padding 2 (fp32 tensors).
//
// A 2x2 output tile of a 5x5 correlation is  A^T [ (G g G^T) (.) (B^T d B) ] A  over its 6x6 input
// patch d, with the interpolation points 0, +-1, +-2 and infinity: 36 multiplications instead of 100
// per tile and channel pair.  B^T is the input transform of any minimal algorithm on these six
// points (it is the one F(4x4,3x3) uses), G (6x5) evaluates the filter polynomial at the points with
// the usual normalisation 1/4, -1/6, -1/6, 1/24, 1/24, 1, and A^T (2x6) = [1 1 1 1 1 0; 0 1 -1 2 -2 1].
//
// The structure is that of wino_fused_kernel (F(2x2,3x3)): the only workspace is the transformed
// filter U[36][Ci8][Co4]; a workgroup owns 64 output channels x 64 tiles, each wave 32 x 32.  36
// accumulator tiles do not fit a wave's registers, so the workgroup makes three passes over the
// input channels, one per pair of rows of the 6x6 point grid (12 points, 192 accumulator
// registers): a pass fetches the patches again, computes the two rows of B^T d B it needs, and at
// its end folds its 12 accumulators into the 2x2 outputs, which stay in registers until the last
// pass (A^T M A is a sum over the rows of M, so the passes' contributions simply add).
// Patch rows are fetched as 16-byte windows starting at column 2*tw (never before the tensor);
// the patch's first two columns are the first two window elements of the tile to the left, taken
// from the lane below with two cross-lane moves (lane 0 fetches them itself, tiles in the first
// tile column take 0), and window elements past the end of the row are replaced by 0.
#include <hip/hip_runtime.h>

#include "gemm_launch.hpp"
#include "kernels.h"

namespace ucd {

namespace {

constexpr int kW5K = 64, kW5T = 64, kW5C = 8;   // block: output channels x tiles; input channels per step
constexpr int kW5Rows = 2;                       // rows of the 6x6 point grid per pass
constexpr int kW5Pts = 6 * kW5Rows;              // points (accumulator tiles) per pass
constexpr int kW5Passes = 6 / kW5Rows;
constexpr int kW5NP = kW5C / 4;                  // patches per thread and step (channel = wave + 4h)
constexpr int kW5NU = kW5Pts * kW5C * kW5K / 4 / 256;   // float4 pieces of a step's U slice per thread
constexpr int kW5Pairs = kW5C / 2;

struct Wino5Params {
    const float *in;
    const float *U;
    float *out;
    uint32_t in_bytes, u_bytes;
    int Ci, Co, Hi, Wi, Ho, Wo, pad_h;
    int T, TW, Mo4, ci_pad;
    FastDiv divT, divTW;
    int n_tiles, k_blocks;
};

struct Geom5 {
    int Ci, Co, Hi, Wi, Ho, Wo, pad_h, pad_w, TH, TW, T, Mo4, ci_pad;
    bool transposed;
};

Geom5 geom5(const Dims &d, int op)
{
    Geom5 g;
    if (op == 0) {
        g.Ci = d.C; g.Co = d.K; g.Hi = d.H; g.Wi = d.W; g.Ho = d.P; g.Wo = d.Q;
        g.pad_h = d.ph; g.pad_w = d.pw; g.transposed = false;
    } else {
        g.Ci = d.K; g.Co = d.C; g.Hi = d.P; g.Wi = d.Q; g.Ho = d.H; g.Wo = d.W;
        g.pad_h = 4 - d.ph; g.pad_w = 4 - d.pw; g.transposed = true;
    }
    g.TH = (g.Ho + 1) / 2; g.TW = (g.Wo + 1) / 2; g.T = g.TH * g.TW;
    g.Mo4 = (g.Co + 3) / 4 * 4;
    g.ci_pad = (g.Ci + kW5C - 1) / kW5C * kW5C;
    return g;
}

// one row of B^T applied to six values
template <int I>
__device__ __forceinline__ float bt_row(float d0, float d1, float d2, float d3, float d4, float d5)
{
    if constexpr (I == 0) return fmaf(-5.f, d2, fmaf(4.f, d0, d4));
    if constexpr (I == 1) return fmaf(-4.f, d1 + d2, d3 + d4);
    if constexpr (I == 2) return fmaf(4.f, d1 - d2, d4 - d3);
    if constexpr (I == 3) return fmaf(2.f, d3 - d1, d4 - d2);
    if constexpr (I == 4) return fmaf(-2.f, d3 - d1, d4 - d2);
    return fmaf(-5.f, d3, fmaf(4.f, d1, d5));
}

// U[xi][ci][co] = (G g G^T)[xi] of the 5x5 filter of (co, ci); planes of Cpad rows (zero past Ci)
__global__ __launch_bounds__(256) void wino5_filter_kernel(const float *__restrict__ w, float *__restrict__ U, int Ci,
                                                           int Co, int Mo4, int transposed, int Cpad)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= Cpad * Mo4) return;
    const int ci = i / Mo4, co = i - ci * Mo4;
    const bool live = co < Co && ci < Ci;
    // G = diag(1/4, -1/6, -1/6, 1/24, 1/24, 1) . [p^k], points 0, 1, -1, 2, -2, infinity
    auto apply_g = [](const float (&g)[5], float (&u)[6]) {
        const float e = g[0] + g[2] + g[4], o = g[1] + g[3];
        const float e2 = g[0] + 4.f * g[2] + 16.f * g[4], o2 = 2.f * g[1] + 8.f * g[3];
        u[0] = 0.25f * g[0];
        u[1] = (-1.f / 6.f) * (e + o);
        u[2] = (-1.f / 6.f) * (e - o);
        u[3] = (1.f / 24.f) * (e2 + o2);
        u[4] = (1.f / 24.f) * (e2 - o2);
        u[5] = g[4];
    };
    float t[6][5];  // G g, column by column
#pragma unroll
    for (int s = 0; s < 5; ++s) {
        float g[5], u[6];
#pragma unroll
        for (int r = 0; r < 5; ++r) {
            float v = 0.f;
            if (live)
                v = transposed ? w[((size_t)(ci * Co + co) * 5 + (4 - r)) * 5 + (4 - s)]
                               : w[((size_t)(co * Ci + ci) * 5 + r) * 5 + s];
            g[r] = v;
        }
        apply_g(g, u);
#pragma unroll
        for (int r = 0; r < 6; ++r) t[r][s] = u[r];
    }
    const size_t plane = (size_t)Cpad * Mo4;
#pragma unroll
    for (int r = 0; r < 6; ++r) {
        float u[6];
        apply_g(t[r], u);
#pragma unroll
        for (int s = 0; s < 6; ++s) U[(size_t)(r * 6 + s) * plane + i] = u[s];
    }
}

template <bool ODD_W>
__global__ __launch_bounds__(256) void wino5_fused_kernel(Wino5Params p)
{
    __shared__ __attribute__((aligned(16))) float Us[2][kW5Pts][kW5C][kW5K];
    __shared__ __attribute__((aligned(16))) float Vs[2][kW5Pts][kW5C][kW5T];
    // the thread's 64 outputs (16 accumulator registers x 2x2) between the passes: value v of thread t at
    // Ys[v][t], so that a wave's accesses are contiguous
    __shared__ float Ys[64][256];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int wk = wave & 1, wt = wave >> 1;

    // consecutive work items of an XCD share a tile block (the input patches) and differ in the channel block
    const uint32_t v = xcd_order(blockIdx.x, gridDim.x);
    const int kb = (int)(v % (uint32_t)p.k_blocks), tb = (int)(v / (uint32_t)p.k_blocks);
    const int k0 = kb * kW5K, t0 = tb * kW5T;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc_bytes(p.in, 0, p.in_bytes);
    const __amdgpu_buffer_rsrc_t ru = make_rsrc_bytes(p.U, 0, p.u_bytes);

    // producer role: the 6x6 patch of tile `lane` of the block, for channels wave, wave + 4 of the step.
    // voff[r]: the 16-byte window of patch row r (columns 2tw .. 2tw+3 = patch columns 2..5);
    // xoff[r]: patch columns 0, 1 of that row, fetched by lane 0 only (the other lanes get them from
    // the lane below)
    uint32_t voff[6], xoff[6];
    bool first_col, ok1, ok2, ok3;
    {
        const int j = t0 + lane;
        uint32_t n = 0, t, th = 0, tw = 0;
        const bool live = j < p.n_tiles;
        if (live) {
            p.divT.divmod((uint32_t)j, n, t);
            p.divTW.divmod(t, th, tw);
        }
        const int h0 = 2 * (int)th - p.pad_h, ws = 2 * (int)tw;
        first_col = tw == 0;
        ok1 = ws + 1 < p.Wi; ok2 = ws + 2 < p.Wi; ok3 = ws + 3 < p.Wi;
#pragma unroll
        for (int r = 0; r < 6; ++r) {
            const int h = h0 + r;
            const bool ok = live && (unsigned)h < (unsigned)p.Hi;
            const uint32_t row = 4u * (uint32_t)(((int)n * p.Ci * p.Hi + h) * p.Wi + ws);
            voff[r] = ok ? row : kOob;
            xoff[r] = ok && lane == 0 && tw > 0 ? row - 8u : kOob;
        }
    }
    // U slice of a step and pass: kW5Pts points x kW5C channels x 64 output channels, as float4: piece id =
    // tid + 256*i -> row = id / 16 = point * kW5C + channel, 4 output channels from 4 * (id % 16); the
    // step's and the pass's parts of the address are a scalar offset
    uint32_t uoff[kW5NU];
#pragma unroll
    for (int i = 0; i < kW5NU; ++i) {
        const int id = tid + 256 * i, row = id >> 4, q = id & 15;
        const int xi = row / kW5C, c = row % kW5C, k = k0 + 4 * q;
        uoff[i] = k < p.Mo4 ? 4u * (uint32_t)((xi * p.ci_pad + c) * p.Mo4 + k) : kOob;
    }
    const int u_slot = (tid >> 4) * kW5K + 4 * (tid & 15);

    float d[kW5NP][36];   // the thread's patches of the step after the one in LDS, as loaded
    f32x4 uq[kW5NU];      // and its share of that step's U slice
    auto chan_off = [&](int c0, int h) {
        const int c = c0 + wave + 4 * h;
        return c < p.Ci ? 4u * (uint32_t)(c * p.Hi * p.Wi) : kOob;   // past the last channel: out of range
    };
    constexpr int kPatchLoads = 12;   // per row: the window, and lane 0's first two columns
    auto fetch_piece = [&](int c0, int h, int i) {
        const uint32_t so = chan_off(c0, h);
        if (i < 6) {
            const f32x4 q = buf_load4(rin, voff[i], so);
            d[h][6 * i + 2] = q.x; d[h][6 * i + 3] = q.y; d[h][6 * i + 4] = q.z; d[h][6 * i + 5] = q.w;
        } else {
            const auto q = __builtin_amdgcn_raw_buffer_load_b64(rin, (int)xoff[i - 6], (int)so, 0);
            d[h][6 * (i - 6)] = __uint_as_float(q[0]);
            d[h][6 * (i - 6) + 1] = __uint_as_float(q[1]);
        }
    };
    auto fetch_u = [&](int c0, int pass, int i) {
        uq[i] = buf_load4(ru, uoff[i], 4u * (uint32_t)((c0 + pass * kW5Pts * p.ci_pad) * p.Mo4));
    };
    // rows 2*pass, 2*pass + 1 of B^T d B of patch h into LDS buffer `buf`
    auto store_v = [&](auto PASS, int buf, int h) {
        constexpr int pass = decltype(PASS)::value;
        // B^T d first (the pass's two rows, column by column): the border handling then touches two
        // values per column instead of six.  Columns 2..5 are the window as loaded.
        float tr[kW5Rows][6];
#pragma unroll
        for (int c = 0; c < 6; ++c) {
            tr[0][c] = bt_row<2 * pass>(d[h][c], d[h][6 + c], d[h][12 + c], d[h][18 + c], d[h][24 + c], d[h][30 + c]);
            tr[1][c] = bt_row<2 * pass + 1>(d[h][c], d[h][6 + c], d[h][12 + c], d[h][18 + c], d[h][24 + c], d[h][30 + c]);
        }
#pragma unroll
        for (int i = 0; i < kW5Rows; ++i) {
            // window elements past the end of the row belong to the next row: their column counts as 0.
            // With an even width the second element is always inside.
            if constexpr (ODD_W) tr[i][3] = ok1 ? tr[i][3] : 0.f;
            tr[i][4] = ok2 ? tr[i][4] : 0.f;
            tr[i][5] = ok3 ? tr[i][5] : 0.f;
            // columns 0, 1 = the first two window columns of the tile to the left: wave_shr:1 takes them
            // from the lane below (lane 0 keeps what it computed from its own loads).  Tiles in the first
            // tile column take 0; with an odd width their left neighbour's second column has just been zeroed.
            const int l0 = __builtin_amdgcn_update_dpp((int)__float_as_uint(tr[i][0]), (int)__float_as_uint(tr[i][2]), 0x138, 0xf, 0xf, false);
            const int l1 = __builtin_amdgcn_update_dpp((int)__float_as_uint(tr[i][1]), (int)__float_as_uint(tr[i][3]), 0x138, 0xf, 0xf, false);
            tr[i][0] = first_col ? 0.f : __uint_as_float((uint32_t)l0);
            tr[i][1] = ODD_W ? __uint_as_float((uint32_t)l1) : first_col ? 0.f : __uint_as_float((uint32_t)l1);
        }
#pragma unroll
        for (int i = 0; i < kW5Rows; ++i) {
            const float *t = tr[i];
            Vs[buf][6 * i + 0][wave + 4 * h][lane] = bt_row<0>(t[0], t[1], t[2], t[3], t[4], t[5]);
            Vs[buf][6 * i + 1][wave + 4 * h][lane] = bt_row<1>(t[0], t[1], t[2], t[3], t[4], t[5]);
            Vs[buf][6 * i + 2][wave + 4 * h][lane] = bt_row<2>(t[0], t[1], t[2], t[3], t[4], t[5]);
            Vs[buf][6 * i + 3][wave + 4 * h][lane] = bt_row<3>(t[0], t[1], t[2], t[3], t[4], t[5]);
            Vs[buf][6 * i + 4][wave + 4 * h][lane] = bt_row<4>(t[0], t[1], t[2], t[3], t[4], t[5]);
            Vs[buf][6 * i + 5][wave + 4 * h][lane] = bt_row<5>(t[0], t[1], t[2], t[3], t[4], t[5]);
        }
    };
    auto store_u = [&](int buf, int i) {
        *reinterpret_cast<f32x4 *>(&Us[buf][0][0][0] + u_slot + 1024 * i) = uq[i];
    };

    auto run_pass = [&](auto PASS) {
        constexpr int pass = decltype(PASS)::value;
        f32x16 acc[kW5Pts];
#pragma unroll
        for (int i = 0; i < kW5Pts; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

        // step 0 -> LDS buffer 0, step 1 -> registers
#pragma unroll
        for (int h = 0; h < kW5NP; ++h)
#pragma unroll
            for (int i = 0; i < kPatchLoads; ++i) fetch_piece(0, h, i);
#pragma unroll
        for (int i = 0; i < kW5NU; ++i) fetch_u(0, pass, i);
#pragma unroll
        for (int h = 0; h < kW5NP; ++h) store_v(PASS, 0, h);
#pragma unroll
        for (int i = 0; i < kW5NU; ++i) store_u(0, i);
#pragma unroll
        for (int h = 0; h < kW5NP; ++h)
#pragma unroll
            for (int i = 0; i < kPatchLoads; ++i) fetch_piece(kW5C, h, i);
#pragma unroll
        for (int i = 0; i < kW5NU; ++i) fetch_u(kW5C, pass, i);
        __syncthreads();

        int buf = 0;
        for (int c0 = 0; c0 < p.Ci; c0 += kW5C) {
            const float *ua = &Us[buf][0][lhi][wk * 32 + l32];
            const float *vb = &Vs[buf][0][lhi][wt * 32 + l32];
            // operands in units of two channel pairs, kAhead units before their MFMAs
            constexpr int kUnits = kW5Pts * kW5Pairs / 2, kAhead = 3;
            float a[kAhead + 1][2], b[kAhead + 1][2];
            auto read_unit = [&](int u) {
                const int xi = u / (kW5Pairs / 2), q0 = 2 * (u % (kW5Pairs / 2));
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    a[u % (kAhead + 1)][q] = ua[(xi * kW5C + 2 * (q0 + q)) * kW5K];
                    b[u % (kAhead + 1)][q] = vb[(xi * kW5C + 2 * (q0 + q)) * kW5T];
                }
            };
#pragma unroll
            for (int u = 0; u < kAhead; ++u) read_unit(u);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(UCD_MFMA_PRIO);
            constexpr int kMfmas = kW5Pts * kW5Pairs;
            // one MFMA and the piece of the step's memory and transform work dealt out behind it (at most
            // one global load per MFMA: a burst would block this SIMD's only wave)
            auto slot = [&](auto M) {
                constexpr int m = decltype(M)::value;
                constexpr int xi = m / kW5Pairs, u = m / 2;
                acc[xi] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u % (kAhead + 1)][m % 2], b[u % (kAhead + 1)][m % 2], acc[xi], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (m % 2 == 0 && u + kAhead < kUnits) read_unit(u + kAhead);
                constexpr int kPatchSlots = 1 + kPatchLoads;
                if constexpr (m >= 1 && m < 1 + kPatchSlots * kW5NP) {
                    constexpr int h = (m - 1) / kPatchSlots, i = (m - 1) % kPatchSlots;
                    if constexpr (i == 0) store_v(PASS, buf ^ 1, h);
                    else fetch_piece(c0 + 2 * kW5C, h, i - 1);
                }
                constexpr int kUStart = 1 + kPatchSlots * kW5NP;
                if constexpr (m >= kUStart && m < kUStart + 2 * kW5NU) {
                    constexpr int i = (m - kUStart) / 2;
                    if constexpr ((m - kUStart) % 2 == 0) store_u(buf ^ 1, i);
                    else fetch_u(c0 + 2 * kW5C, pass, i);
                }
                static_assert(kUStart + 2 * kW5NU <= kMfmas, "the step's work fits behind its MFMAs");
                __builtin_amdgcn_sched_barrier(0);
            };
            static_for<kMfmas>(slot);
            __builtin_amdgcn_s_setprio(0);
            __syncthreads();
            buf ^= 1;
        }

        // Y += A^T[:, i] (M[i][.] A) for the pass's rows i of M, A^T = [1 1 1 1 1 0; 0 1 -1 2 -2 1]; the
        // running sums live in LDS between the passes, the last pass stores the tile
        constexpr float at1[6] = {0.f, 1.f, -1.f, 2.f, -2.f, 1.f};
        constexpr bool last = pass == kW5Passes - 1;
        const int j = t0 + wt * 32 + l32;
        uint32_t n = 0, t, th = 0, tw = 0;
        if (last && j < p.n_tiles) {
            p.divT.divmod((uint32_t)j, n, t);
            p.divTW.divmod(t, th, tw);
        }
        const int ho = 2 * (int)th, wo = 2 * (int)tw;
        const bool h1 = ho + 1 < p.Ho, w1 = wo + 1 < p.Wo;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float y[4] = {0.f, 0.f, 0.f, 0.f};
            if constexpr (pass > 0) {
#pragma unroll
                for (int o = 0; o < 4; ++o) y[o] = Ys[4 * e + o][tid];
            }
#pragma unroll
            for (int ii = 0; ii < kW5Rows; ++ii) {
                constexpr int unused = 0;
                (void)unused;
                const int i = kW5Rows * pass + ii;
                const float m0 = acc[6 * ii][e], m1 = acc[6 * ii + 1][e], m2 = acc[6 * ii + 2][e];
                const float m3 = acc[6 * ii + 3][e], m4 = acc[6 * ii + 4][e], m5 = acc[6 * ii + 5][e];
                const float r0 = (m0 + m1) + (m2 + m3) + m4;
                const float r1 = (m1 - m2) + 2.f * (m3 - m4) + m5;
                if (i < 5) {
                    y[0] += r0;
                    y[1] += r1;
                }
                if (i > 0) {
                    y[2] = fmaf(at1[i], r0, y[2]);
                    y[3] = fmaf(at1[i], r1, y[3]);
                }
            }
            if constexpr (!last) {
#pragma unroll
                for (int o = 0; o < 4; ++o) Ys[4 * e + o][tid] = y[o];
            } else {
                // lane = tile (column l32 of the wave's 32), register e = channel row
                const int k = k0 + wk * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
                if (j < p.n_tiles && k < p.Co) {
                    float *dst = p.out + (((long)n * p.Co + k) * p.Ho + ho) * p.Wo + wo;
                    dst[0] = y[0];
                    if (w1) dst[1] = y[1];
                    if (h1) {
                        dst[p.Wo] = y[2];
                        if (w1) dst[p.Wo + 1] = y[3];
                    }
                }
            }
        }
    };
    run_pass(std::integral_constant<int, 0>{});
    run_pass(std::integral_constant<int, 1>{});
    run_pass(std::integral_constant<int, 2>{});
}


// ---- BackwardFilter: F(5x5,2x2) with both data transforms fused ------------------------------------
// dw (5x5) = G^T [ sum over tiles (A dy A^T) (.) (B^T x B) ] G with A = (A^T)^T (6x2): a 2x2 tile of
// dy and its 6x6 patch of x give 36 products per channel pair.  The workspace holds the 36 K x C
// planes Mw.  As in wino_fused_filter_kernel a workgroup owns a block of output channels x input
// channels and reduces over 8 tile positions of the image (fixed for the workgroup) times a range of
// images, one image per step; here it also owns one pair of rows of the point grid (12 planes), so
// three workgroups share every chunk.  The block is 64 x 64 channels (KW = 2: the waves 2 x 2) or 128
// output x 32 input channels (KW = 4: the waves 4 x 1): transforming a patch of x costs five times
// what a tile of dy costs, so the narrow block halves the vector work per MFMA, and it fits channel
// counts such as 96 that fill one and a half 64-wide blocks.  Patch rows of x are fetched as 16-byte
// windows starting at column 2*tw, the patch's first two columns come from the lane below (the tile
// to the left, same channel) or, for the first tile position of a group, from a load of its own; tile
// rows of dy as 8-byte loads.
constexpr int kF5T = 8, kF5Pairs = kF5T / 2;

struct Wino5FilterParams {
    const float *x, *dy;
    float *Mw;
    uint32_t x_bytes, dy_bytes;
    int C, K, H, W, P, Q, pad_h, T, TW;
    int b, k_blocks, c_blocks, groups, images_per_chunk;
};

template <bool ODD_W, int KW>
__global__ __launch_bounds__(256) void wino5_fused_filter_kernel(Wino5FilterParams p)
{
    constexpr int KB = 32 * KW, CB = 32 * (4 / KW);   // output / input channels of the block
    constexpr int NX = CB / 32, NDY = KB / 32;        // patches of x / tiles of dy per thread and step
    __shared__ __attribute__((aligned(16))) float Ds[2][kW5Pts][kF5T][KB];
    __shared__ __attribute__((aligned(16))) float Vs[2][kW5Pts][kF5T][CB];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int wk = wave % KW, wc = wave / KW;

    // work item: (pass, output-channel block, input-channel block, tile-position group, image chunk);
    // neighbours on an XCD share the x patches and dy tiles
    uint32_t v = xcd_order(blockIdx.x, gridDim.x);
    const int pass = __builtin_amdgcn_readfirstlane((int)(v % (uint32_t)kW5Passes)); v /= (uint32_t)kW5Passes;
    const int kb = (int)(v % (uint32_t)p.k_blocks); v /= (uint32_t)p.k_blocks;
    const int cb = (int)(v % (uint32_t)p.c_blocks); v /= (uint32_t)p.c_blocks;
    const int grp = (int)(v % (uint32_t)p.groups);
    const int chunk = (int)(v / (uint32_t)p.groups);
    const int k0 = kb * KB, c0 = cb * CB;
    const int n_begin = chunk * p.images_per_chunk, n_end = min(p.b, n_begin + p.images_per_chunk);

    const __amdgpu_buffer_rsrc_t rx = make_rsrc_bytes(p.x, 0, p.x_bytes);
    const __amdgpu_buffer_rsrc_t rdy = make_rsrc_bytes(p.dy, 0, p.dy_bytes);

    // producer role: tile position tid % 8 of the group, channel tid / 8 (+ 32 h) of either block; offsets
    // within image 0.  LDS slabs are [point][tile position][channels] with channel c of tile position t
    // at column c ^ 4t (conflict-free stores, operand reads with immediate offsets).
    const int ptile = tid & 7, pch = tid >> 3;
    const int pcol = pch ^ (4 * ptile);
    uint32_t vx[NX][12], vd[NDY][2];   // x: window starts of the 6 patch rows, then this lane's own first columns
    bool own_col, ok1, ok2, ok3, dy_ok1;
    {
        const int t = grp * kF5T + ptile;
        const bool live = t < p.T;
        const int th = live ? t / p.TW : 0, tw = live ? t % p.TW : 0;
        const int h0 = 2 * th - p.pad_h, ws = 2 * tw;
        own_col = ptile == 0 || tw == 0;
        ok1 = ws + 1 < p.W; ok2 = ws + 2 < p.W; ok3 = ws + 3 < p.W;
        dy_ok1 = ws + 1 < p.Q;
#pragma unroll
        for (int h = 0; h < NX; ++h) {
            const int c = c0 + pch + 32 * h;
#pragma unroll
            for (int r = 0; r < 6; ++r) {
                const int hh = h0 + r;
                const bool ok = live && c < p.C && (unsigned)hh < (unsigned)p.H;
                const uint32_t row = 4u * (uint32_t)((c * p.H + hh) * p.W + ws);
                vx[h][r] = ok ? row : kOob;
                vx[h][6 + r] = ok && ptile == 0 && tw > 0 ? row - 8u : kOob;
            }
        }
#pragma unroll
        for (int h = 0; h < NDY; ++h) {
            const int k = k0 + pch + 32 * h;
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int hh = 2 * th + r;
                const bool ok = live && k < p.K && hh < p.P;
                vd[h][r] = ok ? 4u * (uint32_t)((k * p.P + hh) * p.Q + ws) : kOob;
            }
        }
    }
    const uint32_t x_image = 4u * (uint32_t)(p.C * p.H * p.W), dy_image = 4u * (uint32_t)(p.K * p.P * p.Q);

    float dx[NX][36], dz[NDY][4];   // the thread's patches / tiles of the image after the one in LDS, as loaded
    constexpr int kXLoads = 12, kDyLoads = 2;
    // an image past the chunk's end gets a scalar offset that pushes every address out of range
    auto fetch_x = [&](int n, int h, int i) {
        const uint32_t so = n < n_end ? (uint32_t)n * x_image : kOob;
        if (i < 6) {
            const f32x4 q = buf_load4(rx, vx[h][i], so);
            dx[h][6 * i + 2] = q.x; dx[h][6 * i + 3] = q.y; dx[h][6 * i + 4] = q.z; dx[h][6 * i + 5] = q.w;
        } else {
            const auto q = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)vx[h][i], (int)so, 0);
            dx[h][6 * (i - 6)] = __uint_as_float(q[0]);
            dx[h][6 * (i - 6) + 1] = __uint_as_float(q[1]);
        }
    };
    auto fetch_dy = [&](int n, int h, int i) {
        const uint32_t so = n < n_end ? (uint32_t)n * dy_image : kOob;
        const auto q = __builtin_amdgcn_raw_buffer_load_b64(rdy, (int)vd[h][i], (int)so, 0);
        dz[h][2 * i] = __uint_as_float(q[0]);
        dz[h][2 * i + 1] = __uint_as_float(q[1]);
    };
    // rows 2*pass, 2*pass+1 of B^T x B of patch h
    auto store_v = [&](auto PASS, int buf, int h) {
        constexpr int ps = decltype(PASS)::value;
        // B^T x first (the pass's two rows, column by column), then the border handling on two values
        // per column (see wino5_fused_kernel)
        float tr[kW5Rows][6];
#pragma unroll
        for (int c = 0; c < 6; ++c) {
            tr[0][c] = bt_row<2 * ps>(dx[h][c], dx[h][6 + c], dx[h][12 + c], dx[h][18 + c], dx[h][24 + c], dx[h][30 + c]);
            tr[1][c] = bt_row<2 * ps + 1>(dx[h][c], dx[h][6 + c], dx[h][12 + c], dx[h][18 + c], dx[h][24 + c], dx[h][30 + c]);
        }
#pragma unroll
        for (int i = 0; i < kW5Rows; ++i) {
            if constexpr (ODD_W) tr[i][3] = ok1 ? tr[i][3] : 0.f;
            tr[i][4] = ok2 ? tr[i][4] : 0.f;
            tr[i][5] = ok3 ? tr[i][5] : 0.f;
            // the lane below holds the tile to the left (same channel) unless this is the first tile
            // position of the group or of a tile row: then what the lane computed from its own load
            // (0 in the first tile column)
            const int l0 = __builtin_amdgcn_update_dpp(0, (int)__float_as_uint(tr[i][2]), 0x138, 0xf, 0xf, false);
            const int l1 = __builtin_amdgcn_update_dpp(0, (int)__float_as_uint(tr[i][3]), 0x138, 0xf, 0xf, false);
            tr[i][0] = own_col ? tr[i][0] : __uint_as_float((uint32_t)l0);
            tr[i][1] = own_col ? tr[i][1] : __uint_as_float((uint32_t)l1);
        }
#pragma unroll
        for (int i = 0; i < kW5Rows; ++i) {
            const float *t = tr[i];
            Vs[buf][6 * i + 0][ptile][pcol + 32 * h] = bt_row<0>(t[0], t[1], t[2], t[3], t[4], t[5]);
            Vs[buf][6 * i + 1][ptile][pcol + 32 * h] = bt_row<1>(t[0], t[1], t[2], t[3], t[4], t[5]);
            Vs[buf][6 * i + 2][ptile][pcol + 32 * h] = bt_row<2>(t[0], t[1], t[2], t[3], t[4], t[5]);
            Vs[buf][6 * i + 3][ptile][pcol + 32 * h] = bt_row<3>(t[0], t[1], t[2], t[3], t[4], t[5]);
            Vs[buf][6 * i + 4][ptile][pcol + 32 * h] = bt_row<4>(t[0], t[1], t[2], t[3], t[4], t[5]);
            Vs[buf][6 * i + 5][ptile][pcol + 32 * h] = bt_row<5>(t[0], t[1], t[2], t[3], t[4], t[5]);
        }
    };
    // rows 2*pass, 2*pass+1 of A z A^T of tile h, A = [1 0; 1 1; 1 -1; 1 2; 1 -2; 0 1]
    auto store_d = [&](auto PASS, int buf, int h) {
        constexpr int ps = decltype(PASS)::value;
        constexpr float a0[6] = {1.f, 1.f, 1.f, 1.f, 1.f, 0.f}, a1[6] = {0.f, 1.f, -1.f, 2.f, -2.f, 1.f};
        const float z00 = dz[h][0], z01 = ODD_W ? (dy_ok1 ? dz[h][1] : 0.f) : dz[h][1];
        const float z10 = dz[h][2], z11 = ODD_W ? (dy_ok1 ? dz[h][3] : 0.f) : dz[h][3];
#pragma unroll
        for (int ii = 0; ii < kW5Rows; ++ii) {
            const int i = kW5Rows * ps + ii;
            const float t0 = a0[i] * z00 + a1[i] * z10, t1 = a0[i] * z01 + a1[i] * z11;
            Ds[buf][6 * ii + 0][ptile][pcol + 32 * h] = t0;
            Ds[buf][6 * ii + 1][ptile][pcol + 32 * h] = t0 + t1;
            Ds[buf][6 * ii + 2][ptile][pcol + 32 * h] = t0 - t1;
            Ds[buf][6 * ii + 3][ptile][pcol + 32 * h] = fmaf(2.f, t1, t0);
            Ds[buf][6 * ii + 4][ptile][pcol + 32 * h] = fmaf(-2.f, t1, t0);
            Ds[buf][6 * ii + 5][ptile][pcol + 32 * h] = t1;
        }
    };

    int col_q[kF5Pairs];   // the lane's column within its wave's 32, as stored for tile position 2q + lhi
#pragma unroll
    for (int q = 0; q < kF5Pairs; ++q) col_q[q] = l32 ^ (4 * (2 * q + lhi));

    auto run = [&](auto PASS) {
        f32x16 acc[kW5Pts];
#pragma unroll
        for (int i = 0; i < kW5Pts; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

        auto fetch_all = [&](int n) {
#pragma unroll
            for (int h = 0; h < NX; ++h)
#pragma unroll
                for (int i = 0; i < kXLoads; ++i) fetch_x(n, h, i);
#pragma unroll
            for (int h = 0; h < NDY; ++h)
#pragma unroll
                for (int i = 0; i < kDyLoads; ++i) fetch_dy(n, h, i);
        };
        fetch_all(n_begin);
#pragma unroll
        for (int h = 0; h < NX; ++h) store_v(PASS, 0, h);
#pragma unroll
        for (int h = 0; h < NDY; ++h) store_d(PASS, 0, h);
        fetch_all(n_begin + 1);
        __syncthreads();

        int buf = 0;
        for (int n = n_begin; n < n_end; ++n) {
            const float *da = &Ds[buf][0][lhi][wk * 32];
            const float *vb = &Vs[buf][0][lhi][wc * 32];
            float a[2][kF5Pairs], b[2][kF5Pairs];
            auto read_ops = [&](int xi) {
#pragma unroll
                for (int q = 0; q < kF5Pairs; ++q) {
                    a[xi & 1][q] = da[(xi * kF5T + 2 * q) * KB + col_q[q]];
                    b[xi & 1][q] = vb[(xi * kF5T + 2 * q) * CB + col_q[q]];
                }
            };
            read_ops(0);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(UCD_MFMA_PRIO);
            constexpr int kMfmas = kW5Pts * kF5Pairs;
            auto slot = [&](auto M) {
                constexpr int m = decltype(M)::value;
                constexpr int xi = m / kF5Pairs, q = m % kF5Pairs;
                acc[xi] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[xi & 1][q], b[xi & 1][q], acc[xi], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (q == 0 && xi + 1 < kW5Pts) read_ops(xi + 1);
                // image n + 1 (in registers) is transformed into the other LDS buffer and every register
                // reloaded with image n + 2: one piece, at most one global load, behind each MFMA
                constexpr int kXSlots = 1 + kXLoads, kDySlots = 1 + kDyLoads, kDyStart = 1 + NX * kXSlots;
                if constexpr (m >= 1 && m < kDyStart) {
                    constexpr int h = (m - 1) / kXSlots, i = (m - 1) % kXSlots;
                    if constexpr (i == 0) store_v(PASS, buf ^ 1, h);
                    else fetch_x(n + 2, h, i - 1);
                }
                if constexpr (m >= kDyStart && m < kDyStart + NDY * kDySlots) {
                    constexpr int h = (m - kDyStart) / kDySlots, i = (m - kDyStart) % kDySlots;
                    if constexpr (i == 0) store_d(PASS, buf ^ 1, h);
                    else fetch_dy(n + 2, h, i - 1);
                }
                static_assert(kDyStart + NDY * kDySlots <= kMfmas, "the step's work fits behind its MFMAs");
                __builtin_amdgcn_sched_barrier(0);
            };
            static_for<kMfmas>(slot);
            __builtin_amdgcn_s_setprio(0);
            __syncthreads();
            buf ^= 1;
        }

        // lane = input channel (column l32 of the wave's 32), register e = output-channel row
        constexpr int ps = decltype(PASS)::value;
        const int c = c0 + wc * 32 + l32;
        if (c >= p.C) return;
        const size_t plane = (size_t)p.K * p.C;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int k = k0 + wk * 32 + 8 * (e / 4) + 4 * lhi + (e % 4);
            if (k >= p.K) continue;
#pragma unroll
            for (int xi = 0; xi < kW5Pts; ++xi)
                unsafeAtomicAdd(p.Mw + (size_t)(kW5Pts * ps + xi) * plane + (size_t)k * p.C + c, acc[xi][e]);
        }
    };
    if (pass == 0) run(std::integral_constant<int, 0>{});
    else if (pass == 1) run(std::integral_constant<int, 1>{});
    else run(std::integral_constant<int, 2>{});
}

// dw[k, c] (5x5) = beta * dw[k, c] + G^T Mw[., k, c] G, one thread per (k, c)
__global__ __launch_bounds__(256) void wino5_dw_kernel(const float *__restrict__ Mw, float *__restrict__ dw, int KC, float beta)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= KC) return;
    // G^T m for six values m at the points 0, 1, -1, 2, -2, infinity
    auto apply_gt = [](const float (&m)[6], float (&w)[5]) {
        const float s1 = (-1.f / 6.f) * (m[1] + m[2]), d1 = (-1.f / 6.f) * (m[1] - m[2]);
        const float s2 = (1.f / 24.f) * (m[3] + m[4]), d2 = (1.f / 24.f) * (m[3] - m[4]);
        w[0] = 0.25f * m[0] + s1 + s2;
        w[1] = d1 + 2.f * d2;
        w[2] = s1 + 4.f * s2;
        w[3] = d1 + 8.f * d2;
        w[4] = s1 + 16.f * s2 + m[5];
    };
    float tr[5][6];   // G^T Mw, column by column
#pragma unroll
    for (int s = 0; s < 6; ++s) {
        float m[6], w5[5];
#pragma unroll
        for (int r = 0; r < 6; ++r) m[r] = Mw[(size_t)(r * 6 + s) * KC + i];
        apply_gt(m, w5);
#pragma unroll
        for (int r = 0; r < 5; ++r) tr[r][s] = w5[r];
    }
    float *dst = dw + (size_t)i * 25;
#pragma unroll
    for (int r = 0; r < 5; ++r) {
        float w5[5];
        apply_gt(tr[r], w5);
#pragma unroll
        for (int s = 0; s < 5; ++s) dst[r * 5 + s] = beta == 0.f ? w5[s] : beta * dst[r * 5 + s] + w5[s];
    }
}

}  // namespace

bool winograd5_applies(const Dims &d, int op)
{
    if (op < 0 || op > 2) return false;
    if (d.dtype != 0 || d.R != 5 || d.S != 5 || d.sh != 1 || d.sw != 1) return false;
    return d.pw == 2 && d.ph <= 4;   // horizontal padding 2 in both directions (4 - 2 = 2)
}

size_t winograd5_ws_bytes(const Dims &d, int op)
{
    if (op == 2) return (size_t)144 * d.K * d.C;   // the 36 product planes
    const Geom5 g = geom5(d, op);
    return (size_t)144 * g.ci_pad * g.Mo4;
}

hipError_t winograd5_fused(const Dims &d, int op, int b, const void *in, const void *w, void *out, float *ws,
                           bool filter_ready, hipStream_t s)
{
    const Geom5 g = geom5(d, op);
    LaunchLog *log = launch_log();
    if (filter_ready) {
        // U of this filter is still in the workspace from the previous micro-batch
    } else if (log) {
        log->add("wino5_filter_kernel");
    } else {
        wino5_filter_kernel<<<(unsigned)((g.ci_pad * g.Mo4 + 255) / 256), 256, 0, s>>>((const float *)w, ws, g.Ci, g.Co, g.Mo4,
                                                                                     g.transposed ? 1 : 0, g.ci_pad);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    Wino5Params p{};
    p.in = (const float *)in; p.U = ws; p.out = (float *)out;
    p.in_bytes = (uint32_t)(4 * (size_t)b * g.Ci * g.Hi * g.Wi);
    p.u_bytes = (uint32_t)((size_t)144 * g.ci_pad * g.Mo4);
    p.Ci = g.Ci; p.Co = g.Co; p.Hi = g.Hi; p.Wi = g.Wi; p.Ho = g.Ho; p.Wo = g.Wo; p.pad_h = g.pad_h;
    p.T = g.T; p.TW = g.TW; p.Mo4 = g.Mo4; p.ci_pad = g.ci_pad;
    p.divT = FastDiv(g.T); p.divTW = FastDiv(g.TW);
    p.n_tiles = b * g.T;
    p.k_blocks = (g.Co + kW5K - 1) / kW5K;
    const unsigned blocks = (unsigned)(p.k_blocks * ((p.n_tiles + kW5T - 1) / kW5T));
    if (log) {
        log->add("wino5_fused_kernel blocks=" + std::to_string(blocks) + " gemm_flops=" +
                 std::to_string(2.0 * 36 * g.Co * (double)p.n_tiles * g.Ci));
        return hipSuccess;
    }
    if (g.Wi % 2) wino5_fused_kernel<true><<<blocks, 256, 0, s>>>(p);
    else wino5_fused_kernel<false><<<blocks, 256, 0, s>>>(p);
    return hipGetLastError();
}

hipError_t winograd5_fused_filter(const Dims &d, int b, const void *x, const void *dy, float *dw, float beta, float *ws,
                                  hipStream_t s)
{
    const Geom5 g = geom5(d, 0);
    const int KC = d.K * d.C;
    hipError_t e = fill_zero(ws, (size_t)36 * KC, s);
    if (e != hipSuccess) return e;
    Wino5FilterParams p{};
    p.x = (const float *)x; p.dy = (const float *)dy; p.Mw = ws;
    p.x_bytes = xbytes(d, b); p.dy_bytes = ybytes(d, b);
    p.C = d.C; p.K = d.K; p.H = d.H; p.W = d.W; p.P = d.P; p.Q = d.Q; p.pad_h = d.ph; p.T = g.T; p.TW = g.TW;
    p.b = b;
    // block shape: 128 x 32 channels does less vector work per MFMA (one patch of x per thread instead
    // of two); it is taken unless it needs clearly more blocks than 64 x 64
    const long blocks_wide = (long)((d.K + 127) / 128) * ((d.C + 31) / 32), blocks_sq = (long)((d.K + 63) / 64) * ((d.C + 63) / 64);
    const bool wide = blocks_wide * 9 <= blocks_sq * 10;
    p.k_blocks = wide ? (d.K + 127) / 128 : (d.K + 63) / 64;
    p.c_blocks = wide ? (d.C + 31) / 32 : (d.C + 63) / 64;
    p.groups = (g.T + kF5T - 1) / kF5T;
    // image chunks: a workgroup costs its steps plus about 11 steps' worth of start-up and of adding its
    // accumulator tiles into Mw, the launch the rounds of one workgroup per CU times that; the chunk count
    // with the lowest such cost, chunks of at least 4 images
    const long items = (long)kW5Passes * p.k_blocks * p.c_blocks * p.groups, cus = device_cus();
    const long cap = b / 4 < 1 ? 1 : b / 4;
    long split = 1;
    double best = 1e30;
    for (long c = 1; c <= cap && c <= 64; ++c) {
        const int per = (int)((b + c - 1) / c);
        const long wgs = items * ((b + per - 1) / per);
        const double cost = (double)((wgs + cus - 1) / cus) * (per + 11.0);
        if (cost < best - 1e-9) { best = cost; split = c; }
    }
    p.images_per_chunk = (int)((b + split - 1) / split);
    const int n_split = (b + p.images_per_chunk - 1) / p.images_per_chunk;
    const unsigned blocks = (unsigned)(items * n_split);
    LaunchLog *log = launch_log();
    if (log) {
        log->add("wino5_fused_filter_kernel blocks=" + std::to_string(blocks) + " gemm_flops=" +
                 std::to_string(2.0 * 36 * d.K * (double)d.C * p.groups * kF5T * b));
        log->add("wino5_dw_kernel");
        return hipSuccess;
    }
    if (wide) {
        if (d.W % 2) wino5_fused_filter_kernel<true, 4><<<blocks, 256, 0, s>>>(p);
        else wino5_fused_filter_kernel<false, 4><<<blocks, 256, 0, s>>>(p);
    } else {
        if (d.W % 2) wino5_fused_filter_kernel<true, 2><<<blocks, 256, 0, s>>>(p);
        else wino5_fused_filter_kernel<false, 2><<<blocks, 256, 0, s>>>(p);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    wino5_dw_kernel<<<(unsigned)((KC + 255) / 256), 256, 0, s>>>(ws, dw, KC, beta);
    return hipGetLastError();
}

}  // namespace ucd
