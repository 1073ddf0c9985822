// LDS-staged fp32 MFMA tile GEMM for gfx950, with pluggable operand loaders and epilogues.
//
// C[M x N] (+)= A[M x Kd] * B[Kd x N].  One 256-thread workgroup (4 wavefronts of 64) owns a
// BM x BN tile of C and walks Kd in steps of BK = 16.  The operand tiles travel global memory ->
// registers -> one of two LDS buffers laid out [BK][tile + pad] -> v_mfma_f32_32x32x2_f32, as a
// software pipeline two tiles deep whose memory instructions are dealt out behind the MFMAs.
//
// How an operand element (row kk of the reduction, position m in the tile) maps to memory is
// the loader's business: dense matrices, an im2col-style gather from an NCHW tensor, a filter
// gather.  Loaders come in two lane arrangements:
//   * "N-lane": consecutive lanes take consecutive tile positions (coalesced when memory is
//     contiguous along the tile dimension), one reduction row per pass, row index wave-uniform;
//   * "K-lane": consecutive lanes take consecutive reduction indices (coalesced when memory is
//     contiguous along the reduction dimension).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <type_traits>
#include <utility>

namespace ucd {

constexpr int kThreads = 256;
constexpr int kBK = 16;
constexpr int kPad = 4;
#ifndef UCD_MFMA_PRIO
#define UCD_MFMA_PRIO 2
#endif

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Exact n / d for 0 <= n < 2^31 by multiply-high: m = ceil(2^(31+l) / d), l = ceil(log2 d),
// q = mulhi(n, m) >> (l-1).  d = 1 is encoded as m = 0 plus a pass-through mask, so that the
// device code has no branch.
struct FastDiv {
    uint32_t d, m, sh, pass;
    __host__ __device__ FastDiv() : d(1), m(0), sh(0), pass(0xFFFFFFFFu) {}
    __host__ explicit FastDiv(uint32_t div) : d(div), m(0), sh(0), pass(0)
    {
        if (div <= 1) { d = 1; pass = 0xFFFFFFFFu; return; }
        uint32_t l = 0;
        while ((1ull << l) < div) ++l;
        const uint64_t p = 1ull << (31 + l);
        m = (uint32_t)((p + div - 1) / div);
        sh = l - 1;
    }
    __device__ __forceinline__ uint32_t div(uint32_t n) const { return (__umulhi(n, m) >> sh) + (n & pass); }
    __device__ __forceinline__ void divmod(uint32_t n, uint32_t &q, uint32_t &r) const
    {
        q = div(n);
        r = n - q * d;
    }
};

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int WM = BM / (32 * WAVES_M);  // 32x32 MFMA tiles per wave along M
    static constexpr int WN = BN / (32 * WAVES_N);
    static constexpr int LDA = BM + kPad, LDB = BN + kPad;
    static constexpr int LDS_FLOATS = kBK * (LDA + LDB);
    static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
    static_assert(WM >= 1 && WN >= 1, "tile too small for the wave layout");
};

// Block id -> (reduction split, tile).  Workgroups are dealt round-robin to the 8 XCDs by linear
// id (x fastest, then y); this remaps ids so that each XCD (own L2) walks a contiguous range of
// work items ordered split-major, then tile column, then tile row.  Tiles that re-read the same
// B (activation) columns, and all tiles of one reduction chunk (which re-read the same slices of
// both operands), therefore share an L2 instead of pulling the data into all eight.
__device__ __forceinline__ uint32_t xcd_order(uint32_t id, uint32_t total)
{
    const uint32_t xcd = id & 7u, slot = id >> 3;
    const uint32_t q = total >> 3, rem = total & 7u;
    return xcd * q + (xcd < rem ? xcd : rem) + slot;
}
__device__ __forceinline__ void xcd_tile(int tiles_m, int tiles_n, int &tile_m, int &tile_n, int &split)
{
    const uint32_t tiles = (uint32_t)tiles_m * (uint32_t)tiles_n;
    const uint32_t v = xcd_order(blockIdx.x + gridDim.x * blockIdx.y, tiles * gridDim.y);
    split = (int)(v / tiles);
    const uint32_t t = v - (uint32_t)split * tiles;
    tile_m = (int)(t % (uint32_t)tiles_m);
    tile_n = (int)(t / (uint32_t)tiles_m);
}

// Tail spreading.  A launch takes as long as the busiest CU, so a tile count a little above a
// multiple of the CU count costs almost a whole extra round of workgroups.  With `tiles` > 0 the
// reduction steps of the last `tiles` tiles (in tile order), tiles * ksteps of them, are dealt out
// in equal contiguous runs to `wgs` workgroups: a run is a piece of one tile's reduction, or the end
// of one tile's and the start of the next one's.  Each piece is added into a zero-filled output
// with atomics; all other tiles are computed by one workgroup each as usual.
// grid.x = (all tiles - tiles) + wgs, grid.y = 1.
struct TailSplit {
    int tiles, wgs, ksteps;
};

// Loaders may keep per-workgroup state in LDS (`Shared`, filled by `setup` before the main loop,
// one barrier later everybody may read it); most have none.
struct NoShared {};
struct NoSetup {
    typedef NoShared Shared;
    static constexpr bool kHasShared = false;
    static constexpr bool kCellStore = false;  // see GatherNLaneT
    template <class Peer>
    __device__ __forceinline__ void setup(Shared &, int, int, const Peer &) {}
};

// ---- operand loaders ---------------------------------------------------------------------------
// Common interface:  init(params, tile_origin, extent)  once per workgroup;
//                    prep(k0, k_end, peer)   per-step state for reduction rows [k0, k0+BK);
//                    load(i, regs)           global -> register, element i of the thread's NE
//                                            (called for i = 0 .. NE-1 in order, once per step);
//                    store(lds_tile, i, regs) register -> LDS tile laid out [BK][LD].
// Any k0 is legal: rows at or past k_end read as 0 (the main loop prefetches two tiles ahead and
// does not special-case the end of the reduction).
// Elements outside [0, extent) x [0, k_end) read as 0.  All global reads are raw buffer loads
// through a resource that spans exactly the operand (`bytes`): an element that must read as 0
// gets the byte offset kOob, which the hardware range check turns into 0 without touching
// memory.  That keeps the loads branch-free so that they can be issued back to back.  Operands
// are therefore limited to 2 GiB each (checked on the host).

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order: a loop whose index is a
// compile-time constant in every iteration
template <int N, class F>
__device__ __forceinline__ void static_for(F &f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

constexpr uint32_t kOob = 0x80000000u;

// 16 bytes at byte_off + scalar_off (the range check covers the sum)
__device__ __forceinline__ f32x4 buf_load4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, uint32_t scalar_off = 0)
{
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, (int)scalar_off, 0);
    f32x4 v;
    v.x = __uint_as_float(q.x); v.y = __uint_as_float(q.y); v.z = __uint_as_float(q.z); v.w = __uint_as_float(q.w);
    return v;
}

// Element types of tensor operands.  fp32, or bf16 storage: a bf16 value is widened on load by
// placing its 16 bits in the upper half of a register (that is its exact fp32 value, so all
// arithmetic downstream is the fp32 path's) and rounded to nearest-even when an output is stored.
struct bf16 {};
template <class E> struct Elem;
template <> struct Elem<float> {
    static constexpr uint32_t kBytes = 4;
    static const char *tag() { return ""; }
    static __device__ __forceinline__ float load(__amdgpu_buffer_rsrc_t r, uint32_t vo, uint32_t so)
    {
        return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)vo, (int)so, 0));
    }
    static __device__ __forceinline__ void store(void *base, long idx, float v) { ((float *)base)[idx] = v; }
    static __device__ __forceinline__ float get(const void *base, size_t idx) { return ((const float *)base)[idx]; }
};
template <> struct Elem<bf16> {
    static constexpr uint32_t kBytes = 2;
    static const char *tag() { return "/bf16"; }
    static __device__ __forceinline__ float load(__amdgpu_buffer_rsrc_t r, uint32_t vo, uint32_t so)
    {
        const uint32_t h = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)vo, (int)so, 0);
        return __uint_as_float(h << 16);
    }
    static __device__ __forceinline__ uint16_t round(float v)
    {
        const uint32_t u = __float_as_uint(v);
        const uint32_t r = u + 0x7fffu + ((u >> 16) & 1u);  // nearest, ties to even
        return (uint16_t)((v != v ? 0x7fc00000u : r) >> 16);
    }
    static __device__ __forceinline__ void store(void *base, long idx, float v) { ((uint16_t *)base)[idx] = round(v); }
    static __device__ __forceinline__ float get(const void *base, size_t idx)
    {
        return __uint_as_float((uint32_t)((const uint16_t *)base)[idx] << 16);
    }
};
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc_bytes(const void *p, long byte_shift, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)((const char *)p - byte_shift), 0, (int)bytes, 0x00020000);
}

// Gather from an NCHW tensor, lanes along the tile dimension.  Tile position j decodes to
// (n, a, b) over a grid; reduction row kk decodes to (c, r, s); the element is
// T[n, c, a*mul_h + add_h + dir*r, b*mul_w + add_w + dir*s] when in range.
// Forward's B operand: grid = output pixels, mul = stride, add = -pad, dir = +1, T = x.
// BackwardData's B operand (per stride phase): grid = phase pixels, mul = 1, dir = -1, T = dy.
//
// fp32 MFMA and ordinary vector instructions share the SIMD's issue time on this chip, so the
// per-element work in the main loop is kept to two vector instructions: the address splits into
// a per-thread part (fixed for the whole kernel, in a VGPR), and a per-row part (wave-uniform,
// computed on the scalar unit and passed as the load's scalar offset), and "is this tap inside
// the image for my pixel" is one bit of a per-thread mask computed once per workgroup.
// Both address parts are kept non-negative by pointing the buffer resource `shift` elements
// before the tensor (never dereferenced there: every in-range element lies inside the tensor).
struct GatherParams {
    const void *t;
    uint32_t bytes;
    int Ct, Ht, Wt;          // tensor channel count and plane size
    FastDiv grid_hw, grid_w; // tile-position decode
    int mul_h, add_h, mul_w, add_w, dir;
    FastDiv taps, taps_w;    // reduction-row decode: kk -> (c, kk % taps), then (r, s)
    int n_tap_h, n_tap_w;    // taps per axis (R, S of this launch)
    int shift_thread, shift_row;  // elements added to the per-thread / per-row offset parts
};

// SMALL: at most 31 taps, one mask bit per (r, s); otherwise one mask per axis (R, S <= 31).
// NOMASK: every tap of every tile position lies inside the tensor (a layer without padding): the
// per-thread offset is used as it is, and a row past the end of the reduction is pushed out of
// range through the scalar offset: no vector instruction per element at all.
template <int TD, bool SMALL, class E = float, bool NOMASK = false>
struct GatherNLaneT : NoSetup {
    static constexpr uint32_t EB = Elem<E>::kBytes;
    static constexpr bool kBf16 = std::is_same<E, bf16>::value;
    static std::string name() { return std::string(NOMASK ? "GatherNLane<no padding>" : SMALL ? "GatherNLane<taps<=31>" : "GatherNLane<taps>31>") + Elem<E>::tag(); }
    static_assert(TD >= 64, "a wave must cover one reduction row");
    static constexpr int RP = kThreads / TD;  // reduction rows per pass
    static constexpr int NE = kBK / RP;       // elements per thread per step
    static constexpr int LD = TD + kPad;
    // A thread takes a block of NE consecutive rows of the step (NE*row0 + i): their decode is
    // incremental, and in the bf16 kernel the block is a whole run of an LDS cell, written in one piece.
    static constexpr bool kCellStore = kBf16;
    // Where the row decode runs.  With the fp32 matrix pipe every vector instruction costs matrix
    // throughput and the scalar unit is idle: scalar.  With the bf16 pipe the MFMAs are short and
    // the scalar unit, shared by all waves of a CU, becomes the bottleneck: vector lanes.
    static constexpr bool kLaneDecode = kBf16;
    static_assert((NE & (NE - 1)) == 0, "rows per thread: a power of two");
    struct Regs { float r[NE]; };
    const GatherParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t voff;        // per-thread byte offset
    uint32_t nmask, nmask_w;  // bit set = tap outside the image (bit 31 always set)
    int col, row0;
    int k0_, k_end_;
    uint32_t so_v, bit_v, ts_v;     // lane-decoded rows of the step (kLaneDecode)
    uint32_t tap_, tr_, ts_, so_;   // (tap, r, s) and scalar byte offset of the row last loaded
    uint32_t d_tap, e_row, e_chan;  // what that offset grows by per tap, and on top of it when the
                                    // tap starts a new filter row / a new channel

    __device__ __forceinline__ void init(const GatherParams &prm, int origin, int extent)
    {
        p = &prm;
        const int shift = prm.shift_thread + prm.shift_row;
        rsrc = make_rsrc_bytes(prm.t, (long)EB * shift, prm.bytes + EB * (uint32_t)shift);
        tap_ = tr_ = ts_ = so_ = 0;
        so_v = ts_v = 0;
        bit_v = 31;
        d_tap = EB * (uint32_t)prm.dir;
        e_row = EB * (uint32_t)(prm.dir * (prm.Wt - prm.n_tap_w));                  // (r, S-1) -> (r+1, 0)
        e_chan = EB * (uint32_t)(prm.Ht * prm.Wt - prm.dir * prm.n_tap_h * prm.Wt);  // (c, R-1, .) -> (c+1, 0, .)
        const int tid = threadIdx.x;
        col = tid % TD;
        row0 = __builtin_amdgcn_readfirstlane(tid / TD);
        const int j = origin + col;
        nmask = nmask_w = 0xFFFFFFFFu;
        voff = 0;
        if (j < extent) {
            uint32_t n, rest, a, b;
            prm.grid_hw.divmod((uint32_t)j, n, rest);
            prm.grid_w.divmod(rest, a, b);
            const int hb = (int)a * prm.mul_h + prm.add_h, wb = (int)b * prm.mul_w + prm.add_w;
            voff = EB * (uint32_t)((int)n * prm.Ct * prm.Ht * prm.Wt + hb * prm.Wt + wb + prm.shift_thread);
            uint32_t okh = 0, okw = 0;
            for (int r = 0; r < prm.n_tap_h; ++r)
                if ((unsigned)(hb + prm.dir * r) < (unsigned)prm.Ht) okh |= 1u << r;
            for (int q = 0; q < prm.n_tap_w; ++q)
                if ((unsigned)(wb + prm.dir * q) < (unsigned)prm.Wt) okw |= 1u << q;
            if (SMALL) {
                uint32_t ok = 0;
                for (int r = 0; r < prm.n_tap_h; ++r)
                    if ((okh >> r) & 1u) ok |= okw << (r * prm.n_tap_w);
                nmask = ~ok | 0x80000000u;
            } else {
                nmask = ~okh | 0x80000000u;
                nmask_w = ~okw;
            }
        }
    }
    template <class Peer>
    __device__ __forceinline__ void prep(int k0, int k_end, const Peer &)
    {
        k0_ = k0;
        k_end_ = k_end;
        if constexpr (kLaneDecode) {
            // lane i (i < NE) decodes row i of this thread's block; load(i) fetches the result
            // with a read-lane.  All on the vector unit, which has four times the issue slots of
            // the scalar unit the waves of a CU share.
            const int kk = k0 + NE * row0 + (int)(threadIdx.x & (NE - 1));
            uint32_t c, tap, tr, ts;
            p->taps.divmod((uint32_t)kk, c, tap);
            p->taps_w.divmod(tap, tr, ts);
            const bool dead = kk >= k_end;
            so_v = dead ? (NOMASK ? kOob : 0u)
                        : EB * (uint32_t)(((int)c * p->Ht + p->dir * (int)tr) * p->Wt + p->dir * (int)ts + p->shift_row);
            bit_v = dead ? 31u : (SMALL ? tap : tr);
            ts_v = ts;
        }
    }
    // Must be called for i = 0, 1, ..., NE-1 in that order each step: the thread's rows are
    // consecutive, so only the first is decoded by division and the others step the (c, r, s)
    // counters.  Everything up to `so` is wave-uniform and runs on the scalar unit, which all waves
    // of a CU share: with the bf16 matrix pipe the decode, not the MFMAs, sets the pace.
    __device__ __forceinline__ void load(int i, float (&r)[NE])
    {
        if constexpr (kLaneDecode) {
            const uint32_t so = (uint32_t)__builtin_amdgcn_readlane((int)so_v, i);
            const uint32_t bit = (uint32_t)__builtin_amdgcn_readlane((int)bit_v, i);
            uint32_t vo;
            if (NOMASK) {
                vo = voff;
            } else if (SMALL) {
                vo = ((nmask >> bit) << 31) | voff;
            } else {
                const uint32_t ts = (uint32_t)__builtin_amdgcn_readlane((int)ts_v, i);
                vo = (((nmask >> bit) | (nmask_w >> ts)) << 31) | voff;
            }
            r[i] = Elem<E>::load(rsrc, vo, so);
            return;
        }
        const int kk = k0_ + erow(i);
        if (i == 0) {
            uint32_t c;
            p->taps.divmod((uint32_t)kk, c, tap_);
            p->taps_w.divmod(tap_, tr_, ts_);
            so_ = EB * (uint32_t)(((int)c * p->Ht + p->dir * (int)tr_) * p->Wt + p->dir * (int)ts_ + p->shift_row);
        } else {  // one row further: next tap, which may be the next filter row or the next channel
            ++tap_;
            ++ts_;
            const bool row_wrap = ts_ == p->taps_w.d, chan_wrap = tap_ == p->taps.d;  // the second implies the first
            so_ += d_tap + (row_wrap ? e_row : 0u) + (chan_wrap ? e_chan : 0u);
            ts_ = row_wrap ? 0u : ts_;
            tap_ = chan_wrap ? 0u : tap_;
            if (!SMALL) tr_ = chan_wrap ? 0u : tr_ + (row_wrap ? 1u : 0u);
        }
        // wave-uniform by construction; saying so keeps the counters on the scalar unit
        tap_ = (uint32_t)__builtin_amdgcn_readfirstlane((int)tap_);
        ts_ = (uint32_t)__builtin_amdgcn_readfirstlane((int)ts_);
        tr_ = (uint32_t)__builtin_amdgcn_readfirstlane((int)tr_);
        so_ = (uint32_t)__builtin_amdgcn_readfirstlane((int)so_);
        const bool dead = kk >= k_end_;  // rows past the end read as zero
        const uint32_t so = dead ? (NOMASK ? kOob : 0u) : so_;
        uint32_t vo;
        if (NOMASK) {
            vo = voff;
        } else if (SMALL) {
            const uint32_t bit = dead ? 31u : tap_;
            vo = ((nmask >> bit) << 31) | voff;
        } else {
            const uint32_t bit = dead ? 31u : tr_;
            vo = (((nmask >> bit) | (nmask_w >> ts_)) << 31) | voff;
        }
        r[i] = Elem<E>::load(rsrc, vo, so);
    }
    // reduction row (within the step) and tile position of the thread's element i
    __device__ __forceinline__ int erow(int i) const { return NE * row0 + i; }
    __device__ __forceinline__ int ecol(int i) const { return col; }
    __device__ __forceinline__ void store(float *lds, int i, const float (&r)[NE]) const
    {
        lds[erow(i) * LD + col] = r[i];
    }
};
template <int TD> using GatherNLane = GatherNLaneT<TD, true>;
template <int TD> using GatherNLaneBig = GatherNLaneT<TD, false>;
template <int TD> using GatherNLaneFree = GatherNLaneT<TD, false, float, true>;

// ---- loaders with lanes along the reduction dimension -------------------------------------------
// 16 consecutive lanes take the 16 reduction rows of a step for one tile position; a thread owns
// NE = TD/16 tile positions.  Used where memory is contiguous along the reduction index: filter
// matrices, and BackwardFilter's dy / x (contiguous along the pixel index).  The address of
// element (kk, j) is split into a row part computed once per step per thread and a column part
// fixed per thread; wherever the per-element part is the same for the whole wave it is passed as
// the load's scalar offset instead, leaving no per-element vector work (only x in BackwardFilter,
// whose positions decode to irregular (c, r, s), keeps per-element offsets and a window test).
// Rows past k_end get voffset 0x80000000.

struct KLaneParams {
    const void *t;
    uint32_t bytes;
    int row_stride, col_stride;                        // dense: element (kk, j) = t[kk*row_stride + j*col_stride]
    FastDiv taps, taps_w;                              // filter gather: kk -> (k, tap) -> (r, s)
    int k_stride, s_mem, tap_mul_h, tap_add_h, tap_mul_w, tap_add_w, unit_taps;
    FastDiv grid_hw, grid_w, col_taps, col_taps_w;     // pixel rows: kk -> (n, a, b); columns j -> (c, r, s)
    int n_stride, Ht, Wt, mul_h, add_h, mul_w, add_w, shift;
    int n_tap_h, n_tap_w;                              // R, S of the column decode (table loaders)
};

// A note on tile positions outside the operand's extent (the ragged last tile): they only feed
// output rows / columns that the epilogue never stores, so the loaders below do not zero them;
// a buffer load cannot fault, whatever it reads there.  Only the reduction dimension (rows past
// k_end) and genuine padding taps must read as zero.
//
// The hardware range check covers voffset + soffset (probed on the box: a load whose scalar
// offset pushes the sum past num_records returns 0), so the per-element part of an address can
// be a scalar offset whenever it is the same for the whole wave.

// Dense matrix, element (kk, j) = t[kk*row_stride + j*col_stride]  (operand limit 2 GiB).
// One VGPR of address state: the thread's (kl, c0) offset; the step and the position index i enter
// as scalar offsets.
template <int TD, class E = float>
struct KLane0T : NoSetup {
    static constexpr uint32_t EB = Elem<E>::kBytes;
    static constexpr bool kBf16 = std::is_same<E, bf16>::value;
    static std::string name() { return std::string("KLane0") + Elem<E>::tag(); }
    static constexpr int CP = kThreads / kBK;  // tile positions per pass (16)
    static constexpr int NE = TD / CP;
    static constexpr int LD = TD + kPad;
    struct Regs { float r[NE]; };
    const KLaneParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    int kl, c0;
    uint32_t voff;  // byte offset of (row kl, position origin + c0)
    uint32_t vo_;
    int k0_;

    __device__ __forceinline__ void init(const KLaneParams &prm, int origin, int)
    {
        p = &prm;
        rsrc = make_rsrc_bytes(prm.t, 0, prm.bytes);
        kl = threadIdx.x % kBK;
        c0 = threadIdx.x / kBK;
        voff = EB * (uint32_t)(kl * prm.row_stride + (origin + c0) * prm.col_stride);
    }
    template <class Peer>
    __device__ __forceinline__ void prep(int k0, int k_end, const Peer &)
    {
        vo_ = k0 + kl < k_end ? voff : kOob;  // rows past the end read as zero
        k0_ = k0;
    }
    __device__ __forceinline__ void load(int i, float (&r)[NE]) const
    {
        r[i] = Elem<E>::load(rsrc, vo_, EB * (uint32_t)(k0_ * p->row_stride + CP * i * p->col_stride));
    }
    // reduction row (within the step) and tile position of the thread's element i
    __device__ __forceinline__ int erow(int i) const { return kl; }
    __device__ __forceinline__ int ecol(int i) const { return c0 + CP * i; }
    __device__ __forceinline__ void store(float *lds, int i, const float (&r)[NE]) const
    {
        lds[kl * LD + c0 + CP * i] = r[i];
    }
};

template <int TD> using KLane0 = KLane0T<TD, float>;

// BackwardData's A operand: element (kk -> (k, r, s), j = c) = w[k, c, tap_add_h + tap_mul_h*r, tap_add_w + tap_mul_w*s]
// (the filter taps of one stride phase).
template <int TD, class E = float>
struct FilterKLaneT : NoSetup {
    static constexpr uint32_t EB = Elem<E>::kBytes;
    static constexpr bool kBf16 = std::is_same<E, bf16>::value;
    static std::string name() { return std::string("FilterKLane") + Elem<E>::tag(); }
    static constexpr int CP = kThreads / kBK;
    static constexpr int NE = TD / CP;
    static constexpr int LD = TD + kPad;
    struct Regs { float r[NE]; };
    const KLaneParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    int kl, c0;
    uint32_t coff0;  // byte offset of position origin + c0
    uint32_t vo_;

    __device__ __forceinline__ void init(const KLaneParams &prm, int origin, int)
    {
        p = &prm;
        rsrc = make_rsrc_bytes(prm.t, 0, prm.bytes);
        kl = threadIdx.x % kBK;
        c0 = threadIdx.x / kBK;
        coff0 = EB * (uint32_t)((origin + c0) * prm.col_stride);
    }
    template <class Peer>
    __device__ __forceinline__ void prep(int k0, int k_end, const Peer &)
    {
        const int kk = k0 + kl;
        uint32_t k, tap;
        p->taps.divmod((uint32_t)kk, k, tap);
        int roff;
        if (p->unit_taps) {
            roff = (int)k * p->k_stride + (int)tap;
        } else {
            uint32_t tr, ts;
            p->taps_w.divmod(tap, tr, ts);
            roff = (int)k * p->k_stride + (p->tap_add_h + p->tap_mul_h * (int)tr) * p->s_mem + p->tap_add_w +
                   p->tap_mul_w * (int)ts;
        }
        vo_ = kk < k_end ? EB * (uint32_t)roff + coff0 : kOob;
    }
    __device__ __forceinline__ void load(int i, float (&r)[NE]) const
    {
        r[i] = Elem<E>::load(rsrc, vo_, EB * (uint32_t)(CP * i * p->col_stride));
    }
    // reduction row (within the step) and tile position of the thread's element i
    __device__ __forceinline__ int erow(int i) const { return kl; }
    __device__ __forceinline__ int ecol(int i) const { return c0 + CP * i; }
    __device__ __forceinline__ void store(float *lds, int i, const float (&r)[NE]) const
    {
        lds[kl * LD + c0 + CP * i] = r[i];
    }
};

template <int TD> using FilterKLane = FilterKLaneT<TD, float>;

// The same operand with lanes along the tile positions (input channels c, `col_stride` = R*S
// elements apart) and one reduction row per wave and pass: the row part k*k_stride + tap offset is
// wave-uniform and enters as the load's scalar offset.  With 2-byte elements this order costs the
// memory pipeline a third of the cache accesses per load of the reduction-lane loader above
// (measured on 3x3 layers), which is what bounds the bf16 kernel; used for bf16 tensors only.
// No 96-row tile (whole reduction rows per pass).
template <int TD, class E = float>
struct FilterNLaneT : NoSetup {
    static constexpr uint32_t EB = Elem<E>::kBytes;
    static constexpr bool kBf16 = std::is_same<E, bf16>::value;
    static std::string name() { return std::string("FilterNLane") + Elem<E>::tag(); }
    static_assert(kThreads % TD == 0, "whole reduction rows per pass");
    static constexpr bool kUniformRows = TD >= 64;  // a wave stays inside one reduction row
    static constexpr int RP = kThreads / TD;  // reduction rows per pass
    static constexpr int NE = kBK / RP;       // elements per thread per step
    static constexpr int LD = TD + kPad;
    // where the row decode runs: see GatherNLaneT
    static constexpr bool kLaneDecode = kBf16 && kUniformRows;
    struct Regs { float r[NE]; };
    const KLaneParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    int col, row0;
    uint32_t voff;  // byte offset of the thread's tile position
    uint32_t so_v;  // lane i: scalar byte offset of the thread's row i of this step (kLaneDecode)
    int k0_, k_end_;

    __device__ __forceinline__ void init(const KLaneParams &prm, int origin, int)
    {
        p = &prm;
        rsrc = make_rsrc_bytes(prm.t, 0, prm.bytes);
        col = threadIdx.x % TD;
        row0 = kUniformRows ? __builtin_amdgcn_readfirstlane(threadIdx.x / TD) : threadIdx.x / TD;
        // positions past the operand's extent read whatever lies there or zero: never stored
        voff = EB * (uint32_t)((origin + col) * prm.col_stride);
        so_v = kOob;
    }
    // byte offset of reduction row kk = (k, tap), or the "reads as zero" offset past the end
    __device__ __forceinline__ uint32_t row_offset(int kk) const
    {
        uint32_t k, tap;
        p->taps.divmod((uint32_t)kk, k, tap);
        int roff;
        if (p->unit_taps) {
            roff = (int)k * p->k_stride + (int)tap;
        } else {
            uint32_t tr, ts;
            p->taps_w.divmod(tap, tr, ts);
            roff = (int)k * p->k_stride + (p->tap_add_h + p->tap_mul_h * (int)tr) * p->s_mem + p->tap_add_w +
                   p->tap_mul_w * (int)ts;
        }
        return kk < k_end_ ? EB * (uint32_t)roff : kOob;
    }
    template <class Peer>
    __device__ __forceinline__ void prep(int k0, int k_end, const Peer &)
    {
        k0_ = k0;
        k_end_ = k_end;
        if constexpr (kLaneDecode) so_v = row_offset(k0 + row0 + RP * (int)(threadIdx.x & (NE - 1)));
    }
    __device__ __forceinline__ void load(int i, float (&r)[NE]) const
    {
        if constexpr (!kUniformRows) {  // narrow tiles: the row differs within a wave
            const uint32_t ro = row_offset(k0_ + row0 + RP * i);
            r[i] = Elem<E>::load(rsrc, ro == kOob ? kOob : voff + ro, 0);
            return;
        }
        uint32_t so;
        if constexpr (kLaneDecode) so = (uint32_t)__builtin_amdgcn_readlane((int)so_v, i);
        else so = row_offset(k0_ + row0 + RP * i);  // wave-uniform: scalar unit
        r[i] = Elem<E>::load(rsrc, voff, so);
    }
    __device__ __forceinline__ int erow(int i) const { return row0 + RP * i; }
    __device__ __forceinline__ int ecol(int i) const { return col; }
    __device__ __forceinline__ void store(float *lds, int i, const float (&r)[NE]) const
    {
        lds[(row0 + RP * i) * LD + col] = r[i];
    }
};

// BackwardData's A operand when the stride phases of a layer with few input channels are merged
// into one GEMM: the tile position m = (c, a, b) names an input channel and a pixel of a
// (vs_h x vs_w) block of dx (vs = a multiple f of the stride), the reduction row kk = (k, u, v) an
// output channel and a position of the window of dy that reaches the block; the element is
//   w[k, c, a + tap_add_h + tap_mul_h*u, b + tap_add_w + tap_mul_w*v]   (tap_mul = stride,
//   tap_add = -stride*(f-1)), zero where that tap does not exist.
// KLaneParams: col_taps / col_taps_w decode m, taps / taps_w decode kk, n_tap_h / n_tap_w = R, S,
// s_mem = S, col_stride = R*S, k_stride = C*R*S.
template <int TD, class E = float>
struct PhaseFilterKLaneT : NoSetup {
    static constexpr uint32_t EB = Elem<E>::kBytes;
    static constexpr bool kBf16 = std::is_same<E, bf16>::value;
    static std::string name() { return std::string("PhaseFilterKLane") + Elem<E>::tag(); }
    static constexpr int CP = kThreads / kBK;
    static constexpr int NE = TD / CP;
    static constexpr int LD = TD + kPad;
    struct Regs { float r[NE]; };
    const KLaneParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    int kl, c0;
    int coff[NE], rh[NE], rw[NE];  // per position: c*R*S, a + tap_add_h, b + tap_add_w
    int koff_, uh_, vw_;           // per step: k*C*R*S, stride*u, stride*v of this thread's row
    bool live_;

    __device__ __forceinline__ void init(const KLaneParams &prm, int origin, int)
    {
        p = &prm;
        rsrc = make_rsrc_bytes(prm.t, 0, prm.bytes);
        kl = threadIdx.x % kBK;
        c0 = threadIdx.x / kBK;
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            uint32_t c, rest, a, b;
            prm.col_taps.divmod((uint32_t)(origin + c0 + CP * i), c, rest);
            prm.col_taps_w.divmod(rest, a, b);
            coff[i] = (int)c * prm.col_stride;
            rh[i] = (int)a + prm.tap_add_h;
            rw[i] = (int)b + prm.tap_add_w;
        }
    }
    template <class Peer>
    __device__ __forceinline__ void prep(int k0, int k_end, const Peer &)
    {
        const int kk = k0 + kl;
        uint32_t k, tap, u, v;
        p->taps.divmod((uint32_t)kk, k, tap);
        p->taps_w.divmod(tap, u, v);
        koff_ = (int)k * p->k_stride;
        uh_ = p->tap_mul_h * (int)u;
        vw_ = p->tap_mul_w * (int)v;
        live_ = kk < k_end;
    }
    __device__ __forceinline__ void load(int i, float (&r)[NE]) const
    {
        const int tr = rh[i] + uh_, ts = rw[i] + vw_;
        const bool ok = live_ && (unsigned)tr < (unsigned)p->n_tap_h && (unsigned)ts < (unsigned)p->n_tap_w;
        // tile positions past the operand's extent (c >= C) may pass this test: a buffer load
        // cannot fault, and those rows are never stored
        const uint32_t vo = ok ? EB * (uint32_t)(koff_ + coff[i] + tr * p->s_mem + ts) : kOob;
        r[i] = Elem<E>::load(rsrc, vo, 0);
    }
    __device__ __forceinline__ int erow(int i) const { return kl; }
    __device__ __forceinline__ int ecol(int i) const { return c0 + CP * i; }
    __device__ __forceinline__ void store(float *lds, int i, const float (&r)[NE]) const
    {
        lds[kl * LD + c0 + CP * i] = r[i];
    }
};

// BackwardFilter's operands: reduction row kk -> (n, a, b) over the output-pixel grid, tile
// position j -> (c, r, s); element = T[n, c, a*mul_h + add_h + r, b*mul_w + add_w + s].
//   WINDOW = false: dy (a 1x1 "tap", always inside): flags are additive, operand limit 1 GiB.
//   WINDOW = true : x; per step the thread builds, from its pixel, one mask per axis of the taps
//                   that fall outside the image; bit 31 of the row mask is always set and serves
//                   out-of-extent tile positions (r = 31) and rows past the end (mask = all ones).
// The x loader reuses the pixel decode its peer (the dy loader of the same step) has just done.
// NOMASK (x of a layer without padding: every tap of every pixel is inside the image): no masks, one
// address addition per element.
template <int TD, bool WINDOW, class E = float, bool NOMASK = false>
struct PixelKLane : NoSetup {
    static constexpr uint32_t EB = Elem<E>::kBytes;
    static constexpr bool kBf16 = std::is_same<E, bf16>::value;
    static std::string name() { return std::string(!WINDOW ? "PixelKLane<dy>" : NOMASK ? "PixelKLane<x, no padding>" : "PixelKLane<x>") + Elem<E>::tag(); }
    static constexpr int CP = kThreads / kBK;
    static constexpr int NE = TD / CP;
    static constexpr int LD = TD + kPad;
    static constexpr int NV = WINDOW ? NE : 1;
    struct Regs { float r[NE]; };
    const KLaneParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    int kl, c0;
    uint32_t coffb[NV];       // x: byte offset of each position's (c, r, s); dy: of position origin + c0
    uint32_t rs[NV];          // x: r | s << 8
    uint32_t n_, rest_;       // decode of this step's reduction row, for the peer
    uint32_t vo_, nrow_, ncol_;  // this step's row offset and window masks

    __device__ __forceinline__ void init(const KLaneParams &prm, int origin, int extent)
    {
        p = &prm;
        rsrc = make_rsrc_bytes(prm.t, (long)EB * prm.shift, prm.bytes + EB * (uint32_t)prm.shift);
        kl = threadIdx.x % kBK;
        c0 = threadIdx.x / kBK;
        n_ = rest_ = 0;
        if constexpr (!WINDOW) {
            coffb[0] = EB * (uint32_t)((origin + c0) * prm.Ht * prm.Wt);
            rs[0] = 0;
        } else {
#pragma unroll
            for (int i = 0; i < NE; ++i) {
                const int j = origin + c0 + CP * i;
                if (j < extent) {
                    uint32_t c, tap, r, s;
                    prm.col_taps.divmod((uint32_t)j, c, tap);
                    prm.col_taps_w.divmod(tap, r, s);
                    rs[i] = r | (s << 8);
                    coffb[i] = EB * (uint32_t)(((int)c * prm.Ht + (int)r) * prm.Wt + (int)s);
                } else {
                    rs[i] = 31u;  // bit 31 of the row mask is always set
                    coffb[i] = 0u;
                }
            }
        }
    }
    template <class Peer>
    __device__ __forceinline__ void prep(int k0, int k_end, const Peer &peer)
    {
        const int kk = k0 + kl;
        const bool rowok = kk < k_end;
        if constexpr (!WINDOW) {
            p->grid_hw.divmod((uint32_t)kk, n_, rest_);
            // grid is the tensor's own plane here: (a, b) -> a*Wt + b == rest
            vo_ = rowok ? EB * (uint32_t)((int)n_ * p->n_stride + (int)rest_) + coffb[0] : kOob;
        } else {
            uint32_t a, b;
            p->grid_w.divmod(peer.rest_, a, b);
            const int hb = (int)a * p->mul_h + p->add_h, wb = (int)b * p->mul_w + p->add_w;
            vo_ = EB * (uint32_t)((int)peer.n_ * p->n_stride + hb * p->Wt + wb + p->shift);
            if constexpr (NOMASK) {
                vo_ = rowok ? vo_ : kOob;   // + coffb (< 2^31) stays out of range
                return;
            }
            // taps r in [lo, hi) are inside the image; everything else (and bit 31) is masked
            const int lo_h = min(max(-hb, 0), 31), hi_h = max(min(p->Ht - hb, 31), lo_h);
            const int lo_w = min(max(-wb, 0), 31), hi_w = max(min(p->Wt - wb, 31), lo_w);
            const uint32_t nrow = ~(((1u << (hi_h - lo_h)) - 1u) << lo_h);
            ncol_ = ~(((1u << (hi_w - lo_w)) - 1u) << lo_w);
            nrow_ = rowok ? nrow : 0xFFFFFFFFu;
        }
    }
    __device__ __forceinline__ void load(int i, float (&r)[NE]) const
    {
        if constexpr (!WINDOW) {
            const uint32_t step = EB * (uint32_t)(CP * p->Ht * p->Wt);  // scalar: 16 channels further
            r[i] = Elem<E>::load(rsrc, vo_, step * (uint32_t)i);
        } else if constexpr (NOMASK) {
            r[i] = Elem<E>::load(rsrc, vo_ + coffb[i], 0);
        } else {
            const uint32_t t = (nrow_ >> (rs[i] & 0xffu)) | (ncol_ >> (rs[i] >> 8));
            r[i] = Elem<E>::load(rsrc, (t << 31) | (vo_ + coffb[i]), 0);
        }
    }
    // reduction row (within the step) and tile position of the thread's element i
    __device__ __forceinline__ int erow(int i) const { return kl; }
    __device__ __forceinline__ int ecol(int i) const { return c0 + CP * i; }
    __device__ __forceinline__ void store(float *lds, int i, const float (&r)[NE]) const
    {
        lds[kl * LD + c0 + CP * i] = r[i];
    }
};
template <int TD> using DyKLane = PixelKLane<TD, false>;
template <int TD> using XKLane = PixelKLane<TD, true>;
template <int TD> using XKLaneFree = PixelKLane<TD, true, float, true>;

// BackwardFilter's operands again, for filters of at most 31 taps: everything that depends on
// the reduction row alone (the pixel decode, the address
// part of both tensors, and which taps of the window fall outside the image) is computed once per
// workgroup into an LDS table, one entry per row for kTabRows rows at a time (the main loop has
// it refilled when they are used up), instead of once per step per thread.  Per step a thread then reads its entry (two LDS reads for x, one for dy) and spends three
// vector instructions per x element (mask shift, address add, merge) and none per dy element.
constexpr int kTabRows = 1024;
constexpr int kTabCap = kTabRows + 2 * kBK;  // the pipeline looks two steps past the chunk's end

struct PixelTable {
    uint32_t dy_off[kTabCap];   // byte offset of (n, a, b) in dy, or kOob for rows past the end
    uint32_t x_off[kTabCap];    // byte offset of the window origin in x (shifted resource)
    uint32_t tapmask[kTabCap];  // bit r*S+s set = tap outside the image; bit 31 always set
};

template <int TD, class E = float>
struct PixelTabX {
    static constexpr uint32_t EB = Elem<E>::kBytes;
    static constexpr bool kBf16 = std::is_same<E, bf16>::value;
    static std::string name() { return std::string("PixelTab<x>") + Elem<E>::tag(); }
    static constexpr int CP = kThreads / kBK;
    static constexpr int NE = TD / CP;
    static constexpr int LD = TD + kPad;
    typedef PixelTable Shared;
    static constexpr bool kHasShared = true;
    static constexpr bool kCellStore = false;
    struct Regs { float r[NE]; };
    const KLaneParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    const PixelTable *tab;
    int kl, c0, k_begin_;
    uint32_t coffb[NE];   // byte offset of each position's (c, r, s)
    uint32_t tapbit[NE];  // r*S + s, or 31 for positions past the extent
    uint32_t xo_, mask_;  // this step's table entry

    __device__ __forceinline__ void init(const KLaneParams &prm, int origin, int extent)
    {
        p = &prm;
        rsrc = make_rsrc_bytes(prm.t, (long)EB * prm.shift, prm.bytes + EB * (uint32_t)prm.shift);
        kl = threadIdx.x % kBK;
        c0 = threadIdx.x / kBK;
        tab = nullptr;
        k_begin_ = 0;
        xo_ = 0;
        mask_ = 0xFFFFFFFFu;
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            const int j = origin + c0 + CP * i;
            if (j < extent) {
                uint32_t c, tap, r, s;
                prm.col_taps.divmod((uint32_t)j, c, tap);
                prm.col_taps_w.divmod(tap, r, s);
                tapbit[i] = tap;
                coffb[i] = EB * (uint32_t)(((int)c * prm.Ht + (int)r) * prm.Wt + (int)s);
            } else {
                tapbit[i] = 31u;
                coffb[i] = 0u;
            }
        }
    }
    // Fills the table for rows [k_begin, k_begin + kTabCap), k_begin being the start of the chunk
    // or of a later refill: the peer is the dy loader of the same GEMM (its parameters give dy's
    // strides).
    template <class Peer>
    __device__ __forceinline__ void setup(PixelTable &sh, int k_begin, int k_end, const Peer &peer)
    {
        tab = &sh;
        k_begin_ = k_begin;
        const KLaneParams &q = *peer.p;
#pragma unroll 1
        for (int e = threadIdx.x; e < kTabCap; e += kThreads) {
            const int kk = k_begin + e;
            uint32_t n, rest, a, b;
            p->grid_hw.divmod((uint32_t)kk, n, rest);
            p->grid_w.divmod(rest, a, b);
            const int hb = (int)a * p->mul_h + p->add_h, wb = (int)b * p->mul_w + p->add_w;
            uint32_t okw = 0, ok = 0;
#pragma unroll 1
            for (int s = 0; s < p->n_tap_w; ++s)
                if ((unsigned)(wb + s) < (unsigned)p->Wt) okw |= 1u << s;
#pragma unroll 1
            for (int r = 0; r < p->n_tap_h; ++r)
                if ((unsigned)(hb + r) < (unsigned)p->Ht) ok |= okw << (r * p->n_tap_w);
            const bool live = kk < k_end;
            sh.tapmask[e] = live ? (~ok | 0x80000000u) : 0xFFFFFFFFu;
            sh.x_off[e] = EB * (uint32_t)((int)n * p->n_stride + hb * p->Wt + wb + p->shift);
            sh.dy_off[e] = live ? Peer::EB * (uint32_t)((int)n * q.n_stride + (int)rest) : kOob;
        }
    }
    template <class Peer>
    __device__ __forceinline__ void prep(int k0, int, const Peer &)
    {
        const int e = k0 - k_begin_ + kl;
        xo_ = tab->x_off[e];
        mask_ = tab->tapmask[e];
    }
    __device__ __forceinline__ void load(int i, float (&r)[NE]) const
    {
        const uint32_t t = mask_ >> tapbit[i];
        r[i] = Elem<E>::load(rsrc, (t << 31) | (xo_ + coffb[i]), 0);
    }
    // reduction row (within the step) and tile position of the thread's element i
    __device__ __forceinline__ int erow(int i) const { return kl; }
    __device__ __forceinline__ int ecol(int i) const { return c0 + CP * i; }
    __device__ __forceinline__ void store(float *lds, int i, const float (&r)[NE]) const
    {
        lds[kl * LD + c0 + CP * i] = r[i];
    }
};

template <int TD, class E = float>
struct PixelTabDy : NoSetup {
    static constexpr uint32_t EB = Elem<E>::kBytes;
    static constexpr bool kBf16 = std::is_same<E, bf16>::value;
    static std::string name() { return std::string("PixelTab<dy>") + Elem<E>::tag(); }
    static constexpr int CP = kThreads / kBK;
    static constexpr int NE = TD / CP;
    static constexpr int LD = TD + kPad;
    struct Regs { float r[NE]; };
    const KLaneParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    int kl, c0;
    uint32_t coff0;  // byte offset of position origin + c0 (a channel plane)
    uint32_t vo_;

    __device__ __forceinline__ void init(const KLaneParams &prm, int origin, int)
    {
        p = &prm;
        rsrc = make_rsrc_bytes(prm.t, 0, prm.bytes);
        kl = threadIdx.x % kBK;
        c0 = threadIdx.x / kBK;
        coff0 = EB * (uint32_t)((origin + c0) * prm.Ht * prm.Wt);
        vo_ = kOob;
    }
    // the peer is the x loader, whose table holds dy's row offsets as well
    template <class Peer>
    __device__ __forceinline__ void prep(int k0, int, const Peer &peer)
    {
        vo_ = peer.tab->dy_off[k0 - peer.k_begin_ + kl] + coff0;  // kOob + coff0 stays out of range
    }
    __device__ __forceinline__ void load(int i, float (&r)[NE]) const
    {
        const uint32_t step = EB * (uint32_t)(CP * p->Ht * p->Wt);  // scalar: 16 channels further
        r[i] = Elem<E>::load(rsrc, vo_, step * (uint32_t)i);
    }
    // reduction row (within the step) and tile position of the thread's element i
    __device__ __forceinline__ int erow(int i) const { return kl; }
    __device__ __forceinline__ int ecol(int i) const { return c0 + CP * i; }
    __device__ __forceinline__ void store(float *lds, int i, const float (&r)[NE]) const
    {
        lds[kl * LD + c0 + CP * i] = r[i];
    }
};

// Dense matrix contiguous along the tile dimension:  element (kk, j) = t[kk*ld + j], float4 loads.
// Requires ld % 4 == 0 and a 16-byte aligned base; columns in [extent, ld) may hold anything.
struct DenseParams {
    const void *t;
    uint32_t bytes;
    int ld;
};

template <int TD>
struct DenseNLane : NoSetup {
    static constexpr bool kBf16 = false;
    static const char *name() { return "DenseNLane"; }
    static constexpr int CQ = TD / 4;          // float4 columns per row
    static constexpr int RP = kThreads / CQ;   // rows per pass
    static constexpr int NE = (kBK + RP - 1) / RP;
    static constexpr int LD = TD + kPad;
    struct Regs { f32x4 r[NE]; };
    const DenseParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    int col, row0, j_;
    bool ok_;
    int k0_, k_end_;

    __device__ __forceinline__ void init(const DenseParams &prm, int origin, int extent)
    {
        p = &prm;
        rsrc = make_rsrc_bytes(prm.t, 0, prm.bytes);
        const int tid = threadIdx.x;
        col = (tid % CQ) * 4;
        row0 = tid / CQ;
        j_ = origin + col;
        ok_ = j_ < extent;
    }
    template <class Peer>
    __device__ __forceinline__ void prep(int k0, int k_end, const Peer &)
    {
        k0_ = k0;
        k_end_ = k_end;
    }
    __device__ __forceinline__ void load(int i, f32x4 (&r)[NE]) const
    {
        const int row = row0 + RP * i;
        const int kk = k0_ + row;
        const bool ok = ok_ && row < kBK && kk < k_end_;
        r[i] = buf_load4(rsrc, ok ? (uint32_t)(kk * p->ld + j_) * 4u : kOob);
    }
    __device__ __forceinline__ void store(float *lds, int i, const f32x4 (&r)[NE]) const
    {
        const int row = row0 + RP * i;
        if (row < kBK) *reinterpret_cast<f32x4 *>(lds + row * LD + col) = r[i];
    }
};

// Same matrix, any ld / alignment: scalar loads, one reduction row per pass.
template <int TD, class E = float>
struct DenseNLaneST : NoSetup {
    static constexpr uint32_t EB = Elem<E>::kBytes;
    static constexpr bool kBf16 = std::is_same<E, bf16>::value;
    static std::string name() { return std::string("DenseNLaneS") + Elem<E>::tag(); }
    static constexpr int RP = kThreads / TD;
    static constexpr int NE = kBK / RP;
    static constexpr int LD = TD + kPad;
    struct Regs { float r[NE]; };
    const DenseParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    int col, row0, j_;
    bool ok_;
    int k0_, k_end_;

    __device__ __forceinline__ void init(const DenseParams &prm, int origin, int extent)
    {
        p = &prm;
        rsrc = make_rsrc_bytes(prm.t, 0, prm.bytes);
        const int tid = threadIdx.x;
        col = tid % TD;
        row0 = TD >= 64 ? __builtin_amdgcn_readfirstlane(tid / TD) : tid / TD;  // wave-uniform only if TD >= 64
        j_ = origin + col;
        ok_ = j_ < extent;
    }
    template <class Peer>
    __device__ __forceinline__ void prep(int k0, int k_end, const Peer &)
    {
        k0_ = k0;
        k_end_ = k_end;
    }
    __device__ __forceinline__ void load(int i, float (&r)[NE]) const
    {
        const int kk = k0_ + row0 + RP * i;
        r[i] = Elem<E>::load(rsrc, (kk < k_end_ && ok_) ? (uint32_t)(kk * p->ld + j_) * EB : kOob, 0);
    }
    // reduction row (within the step) and tile position of the thread's element i
    __device__ __forceinline__ int erow(int i) const { return row0 + RP * i; }
    __device__ __forceinline__ int ecol(int i) const { return col; }
    __device__ __forceinline__ void store(float *lds, int i, const float (&r)[NE]) const
    {
        lds[(row0 + RP * i) * LD + col] = r[i];
    }
};

template <int TD> using DenseNLaneS = DenseNLaneST<TD, float>;

// The tensor-facing loaders for element type E, as templates of the tile extent alone.
template <class E>
struct Loaders {
    template <int TD> using KLane0 = KLane0T<TD, E>;
    template <int TD> using FilterKLane = FilterKLaneT<TD, E>;
    template <int TD> using PhaseFilterKLane = PhaseFilterKLaneT<TD, E>;
    template <int TD> using FilterNLane = FilterNLaneT<TD, E>;
    template <int TD> using GatherNLane = GatherNLaneT<TD, true, E>;
    template <int TD> using GatherNLaneBig = GatherNLaneT<TD, false, E>;
    template <int TD> using GatherNLaneFree = GatherNLaneT<TD, false, E, true>;
    template <int TD> using DyKLane = PixelKLane<TD, false, E>;
    template <int TD> using XKLane = PixelKLane<TD, true, E>;
    template <int TD> using XKLaneFree = PixelKLane<TD, true, E, true>;
    template <int TD> using DyTab = PixelTabDy<TD, E>;
    template <int TD> using XTab = PixelTabX<TD, E>;
    template <int TD> using DenseNLaneS = DenseNLaneST<TD, E>;
};

// ---- epilogues ---------------------------------------------------------------------------------
// store(m, j, v) for one accumulator element; `prep(j)` decodes a column once for 16 rows.

// Scatter into an NCHW tensor: column j -> (n, a, b) over a (CH x CW) grid, element
// out[n, m, h0 + hs*a, w0 + ws*b].  Forward writes y with the trivial grid; BackwardData writes
// one stride phase of dx.
struct EpiNCHWParams {
    void *out;
    FastDiv grid_hw, grid_w;
    int M, HWo, Wo, h0, hs, w0, ws;
    int cols;  // pixels per image of the column grid when grid_hw divides by a padded count; 0 = no padding
};
template <class E>
struct EpiNCHWT {
    static std::string name() { return std::string("EpiNCHW") + Elem<E>::tag(); }
    typedef EpiNCHWParams Params;
    int off;
    // false: column j is padding (the grid's pixel count may be rounded up past `cols`, see RunNLaneT)
    __device__ __forceinline__ bool prep(const Params &p, int j)
    {
        uint32_t n, rest, a, b;
        p.grid_hw.divmod((uint32_t)j, n, rest);
        p.grid_w.divmod(rest, a, b);
        off = (int)n * p.M * p.HWo + (p.h0 + p.hs * (int)a) * p.Wo + p.w0 + p.ws * (int)b;
        return p.cols == 0 || (int)rest < p.cols;
    }
    __device__ __forceinline__ void store(const Params &p, int m, float v) const
    {
        Elem<E>::store(p.out, off + m * p.HWo, v);
    }
    // accumulate instead of store (tail splitting; fp32 outputs only)
    static constexpr bool kCanAdd = std::is_same<E, float>::value;
    __device__ __forceinline__ void add(const Params &p, int m, float v) const
    {
        unsafeAtomicAdd((float *)p.out + off + m * p.HWo, v);
    }
};
typedef EpiNCHWT<float> EpiNCHW;
// The same scatter as an fp32 atomic add into a zero-filled tensor, for GEMMs whose reduction is
// split over several workgroups because the output has too few tiles to fill the chip.
struct EpiNCHWAtomic : EpiNCHW {
    static constexpr bool kCanAdd = false;
    static const char *name() { return "EpiNCHWAtomic"; }
    __device__ __forceinline__ void store(const Params &p, int m, float v) const
    {
        unsafeAtomicAdd((float *)p.out + off + m * p.HWo, v);
    }
};

// BackwardData with merged stride phases: column j -> (n, t, u) over the grid of (vs_h x vs_w)
// pixel blocks, row m -> (c, a, b); element out[n, c, vs_h*t - pad_h + a, vs_w*u - pad_w + b]
// where that pixel exists.  Every pixel of dx belongs to exactly one (block, position).
struct EpiPhasesParams {
    void *out;
    FastDiv grid_hw, grid_w, block, block_w;
    int C, H, W, vs_h, vs_w, pad_h, pad_w;
};
template <class E>
struct EpiPhasesT {
    static constexpr bool kCanAdd = false;
    static std::string name() { return std::string("EpiPhases") + Elem<E>::tag(); }
    typedef EpiPhasesParams Params;
    int nb, hb, wb;
    __device__ __forceinline__ bool prep(const Params &p, int j)
    {
        uint32_t n, rest, t, u;
        p.grid_hw.divmod((uint32_t)j, n, rest);
        p.grid_w.divmod(rest, t, u);
        nb = (int)n * p.C * p.H * p.W;
        hb = p.vs_h * (int)t - p.pad_h;
        wb = p.vs_w * (int)u - p.pad_w;
        return true;
    }
    __device__ __forceinline__ void store(const Params &p, int m, float v) const
    {
        uint32_t c, rest, a, b;
        p.block.divmod((uint32_t)m, c, rest);
        p.block_w.divmod(rest, a, b);
        const int h = hb + (int)a, w = wb + (int)b;
        if ((unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W)
            Elem<E>::store(p.out, nb + ((int)c * p.H + h) * p.W + w, v);
    }
};

// Dense row-major store out[m*ld + j].
struct EpiDenseParams {
    float *out;
    int ld;
};
struct EpiDense {
    static constexpr bool kCanAdd = false;
    static const char *name() { return "EpiDense"; }
    typedef EpiDenseParams Params;
    int j_;
    __device__ __forceinline__ bool prep(const Params &, int j) { j_ = j; return true; }
    __device__ __forceinline__ void store(const Params &p, int m, float v) const { p.out[(size_t)m * p.ld + j_] = v; }
};

// Dense row-major accumulate with hardware fp32 atomics (split-K partial sums of BackwardFilter).
struct EpiAtomic {
    static constexpr bool kCanAdd = false;
    static const char *name() { return "EpiAtomic"; }
    typedef EpiDenseParams Params;
    int j_;
    __device__ __forceinline__ bool prep(const Params &, int j) { j_ = j; return true; }
    __device__ __forceinline__ void store(const Params &p, int m, float v) const
    {
        unsafeAtomicAdd(p.out + (size_t)m * p.ld + j_, v);
    }
};

// Dense row-major store of one reduction chunk's partial result into that chunk's own plane,
// out + split * plane (the planes are summed in a fixed order by a second kernel: the
// run-to-run reproducible alternative to EpiAtomic).
struct EpiPartialParams {
    float *out;
    int ld;
    long plane;
};
struct EpiPartial {
    static constexpr bool kCanAdd = false;
    static constexpr bool kPerSplit = true;
    static const char *name() { return "EpiPartial"; }
    typedef EpiPartialParams Params;
    int j_;
    __device__ __forceinline__ bool prep(const Params &, int j) { j_ = j; return true; }
    __device__ __forceinline__ void store(const Params &p, int m, float v) const { p.out[(size_t)m * p.ld + j_] = v; }
};
template <class Epi>
__host__ __device__ constexpr auto per_split(int) -> decltype(Epi::kPerSplit) { return Epi::kPerSplit; }
template <class Epi>
__host__ __device__ constexpr bool per_split(...) { return false; }

// What a workgroup computes: a tile and a range of reduction rows (chunk `split`); `accumulate` = it
// adds a partial result (a piece of a tail tile) instead of storing.
struct WorkItem {
    int m0, n0, k_begin, k_end, split;
    bool accumulate;
};
template <class T>
__device__ __forceinline__ WorkItem work_item(int Kd, int k_chunk, int tiles_m, int tiles_n, int whole_tiles)
{
    int tile_m, tile_n, split = 0;
    WorkItem w;
    w.accumulate = false;
    if (whole_tiles > 0) {  // a launch with a spread tail: the tiles in front of it, one workgroup each
        const int t = (int)xcd_order(blockIdx.x, (uint32_t)whole_tiles);
        tile_m = t % tiles_m;
        tile_n = t / tiles_m;
    } else {
        xcd_tile(tiles_m, tiles_n, tile_m, tile_n, split);
    }
    w.m0 = tile_m * T::BM;
    w.n0 = tile_n * T::BN;
    w.k_begin = split * k_chunk;
    w.k_end = min(Kd, w.k_begin + k_chunk);
    w.split = split;
    return w;
}
// The next piece of a tail workgroup's run [it, it_end) of reduction steps, numbered through the
// tail tiles one after another (ksteps each); false when the run is used up.
template <class T>
__device__ __forceinline__ bool next_tail_item(WorkItem &w, int &it, int it_end, int whole_tiles, int ksteps,
                                               int tiles_m, int Kd)
{
    if (it >= it_end) return false;
    const int t = whole_tiles + it / ksteps, s0 = it % ksteps;
    const int s1 = min(ksteps, s0 + (it_end - it));
    w.m0 = (t % tiles_m) * T::BM;
    w.n0 = (t / tiles_m) * T::BN;
    w.k_begin = s0 * kBK;
    w.k_end = min(Kd, s1 * kBK);
    w.accumulate = true;
    w.split = 0;
    it += s1 - s0;
    return true;
}

// Stores (or adds) a wave's accumulators.  Element v of a 32x32 MFMA tile: row
// 8*(v/4) + 4*(lane/32) + v%4, column lane%32.  A wave's WM MFMA tiles along M are interleaved:
// MFMA row r of tile i is wave row WM*r + i, so that a lane's A operands of one reduction row are
// adjacent in LDS and come in one read with an immediate offset.  Columns are not interleaved:
// consecutive lanes must keep consecutive output columns, or every store would touch only every
// other element of a cache line (that cost the bandwidth-bound 1x1 layers a quarter of their speed).
template <class T, class Epi, bool INTERLEAVED = true>
__device__ __forceinline__ void write_tile(const typename Epi::Params &pe, const f32x16 (&acc)[T::WM][T::WN], int M,
                                           int N, int m0, int n0, int wm0, int wn0, int l32, int lhi,
                                           bool accumulate)
{
    Epi epi;
#pragma unroll
    for (int j = 0; j < T::WN; ++j) {
        const int col = n0 + wn0 + j * 32 + l32;
        if (col >= N) continue;
        if (!epi.prep(pe, col)) continue;
#pragma unroll
        for (int i = 0; i < T::WM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r32 = 8 * (v / 4) + 4 * lhi + (v % 4);  // row within the 32x32 MFMA tile
                const int row = m0 + wm0 + (INTERLEAVED ? T::WM * r32 + i : 32 * i + r32);
                if (row < M) {
                    if constexpr (Epi::kCanAdd) {
                        if (accumulate) epi.add(pe, row, acc[i][j][v]);
                        else epi.store(pe, row, acc[i][j][v]);
                    } else {
                        epi.store(pe, row, acc[i][j][v]);
                    }
                }
            }
    }
}

// ---- the kernel --------------------------------------------------------------------------------
// grid.x = tiles_m * tiles_n (XCD-remapped), grid.y = reduction splits (chunk `k_chunk`, a multiple
// of BK), grid.z = batch of independent GEMMs (loaders/epilogue see pointers advanced by the
// given element strides).
template <class T, class ALoader, class BLoader, class Epi, class AParams, class BParams>
__global__ __launch_bounds__(kThreads) void gemm_kernel(AParams pa, BParams pb, typename Epi::Params pe,
                                                         int M, int N, int Kd, int k_chunk, int tiles_m,
                                                         int tiles_n, long a_batch, long b_batch, long c_batch,
                                                         TailSplit tail)
{
    __shared__ __attribute__((aligned(16))) float lds[2][T::LDS_FLOATS];

    if (blockIdx.z) {  // batched GEMMs run on fp32 matrices (strides in floats)
        pa.t = (const float *)pa.t + a_batch * blockIdx.z;
        pb.t = (const float *)pb.t + b_batch * blockIdx.z;
        pe.out = (float *)pe.out + c_batch * blockIdx.z;
    }
    __shared__ typename ALoader::Shared sha;
    __shared__ typename BLoader::Shared shb;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm0 = (wave % T::WAVES_M) * (T::WM * 32);
    const int wn0 = (wave / T::WAVES_M) * (T::WN * 32);
    const int l32 = lane & 31, lhi = lane >> 5;

    // What this workgroup computes: one tile (and reduction chunk), or, in the spread tail of a
    // launch, a run of reduction steps that may end one tile and start the next.
    WorkItem wi;
    int tail_it = 0, tail_end = 0;
    const int whole_tiles = (Epi::kCanAdd && tail.tiles > 0) ? tiles_m * tiles_n - tail.tiles : 0;
    const bool tail_wg = Epi::kCanAdd && tail.tiles > 0 && (int)blockIdx.x >= whole_tiles;
    if (tail_wg) {
        const int r = (int)blockIdx.x - whole_tiles, steps = tail.tiles * tail.ksteps;
        tail_it = (int)((long)r * steps / tail.wgs);
        tail_end = (int)((long)(r + 1) * steps / tail.wgs);
        if (!next_tail_item<T>(wi, tail_it, tail_end, whole_tiles, tail.ksteps, tiles_m, Kd)) return;
    } else {
        wi = work_item<T>(Kd, k_chunk, tiles_m, tiles_n, whole_tiles);
        if constexpr (per_split<Epi>(0)) pe.out += (long)wi.split * pe.plane;
    }
    for (;;) {
        const int m0 = wi.m0, n0 = wi.n0, k_begin = wi.k_begin, k_end = wi.k_end;
        const bool accumulate = wi.accumulate;

        ALoader la;
        BLoader lb;
        la.init(pa, m0, M);
        lb.init(pb, n0, N);
        la.setup(sha, k_begin, k_end, lb);
        lb.setup(shb, k_begin, k_end, la);
        if constexpr (ALoader::kHasShared || BLoader::kHasShared) __syncthreads();

        f32x16 acc[T::WM][T::WN];
#pragma unroll
        for (int i = 0; i < T::WM; ++i)
#pragma unroll
            for (int j = 0; j < T::WN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

        typename ALoader::Regs ra;
        typename BLoader::Regs rb;

        // Software pipeline, two tiles deep with one register set: during step s (MFMAs on tile s from
        // one LDS buffer) the registers holding tile s+1, loaded during step s-1, are written to the
        // other LDS buffer and immediately reloaded with tile s+2.  That work is dealt out over the 8
        // k-pairs of the step, so that each wave always has MFMAs in flight while it issues its loads
        // and LDS writes (a wave that issued them in one block would leave the matrix pipe idle unless
        // another wave happened to be in its MFMA phase).
        constexpr int NA = ALoader::NE, NB = BLoader::NE, kGroups = kBK / 2;
        la.prep(k_begin, k_end, lb);
        lb.prep(k_begin, k_end, la);
#pragma unroll
        for (int i = 0; i < NA; ++i) la.load(i, ra.r);
#pragma unroll
        for (int i = 0; i < NB; ++i) lb.load(i, rb.r);
#pragma unroll
        for (int i = 0; i < NA; ++i) la.store(lds[0], i, ra.r);
#pragma unroll
        for (int i = 0; i < NB; ++i) lb.store(lds[0] + kBK * T::LDA, i, rb.r);
        la.prep(k_begin + kBK, k_end, lb);
        lb.prep(k_begin + kBK, k_end, la);
#pragma unroll
        for (int i = 0; i < NA; ++i) la.load(i, ra.r);
#pragma unroll
        for (int i = 0; i < NB; ++i) lb.load(i, rb.r);
        __syncthreads();

        int buf = 0;
        for (int k0 = k_begin; k0 < k_end; k0 += kBK) {
            if constexpr (ALoader::kHasShared || BLoader::kHasShared) {
                // LDS tables hold kTabRows reduction rows (plus the two tiles of lookahead, already
                // fetched from the old contents): refill them at every multiple of that
                if (k0 != k_begin && ((k0 - k_begin) & (kTabRows - 1)) == 0) {
                    __syncthreads();
                    la.setup(sha, k0, k_end, lb);
                    lb.setup(shb, k0, k_end, la);
                    __syncthreads();
                }
            }
            const float *As = lds[buf];
            const float *Bs = lds[buf] + kBK * T::LDA;
            float *An = lds[buf ^ 1];
            float *Bn = lds[buf ^ 1] + kBK * T::LDA;
            // operands of the next k-pair are read from LDS before the MFMAs of the current one issue
            float a[2][T::WM], b[2][T::WN];
#pragma unroll
            for (int i = 0; i < T::WM; ++i) a[0][i] = As[lhi * T::LDA + wm0 + T::WM * l32 + i];
#pragma unroll
            for (int j = 0; j < T::WN; ++j) b[0][j] = Bs[lhi * T::LDB + wn0 + j * 32 + l32];
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(UCD_MFMA_PRIO);  // a wave inside its MFMA run keeps the pipe
#pragma unroll
            for (int kk = 0; kk < kBK; kk += 2) {
                const int g = kk >> 1, cur = g & 1, nxt = cur ^ 1;
                constexpr int NM = T::WM * T::WN;
                // each piece of memory work issues behind one MFMA, in the shadow of its 16 passes
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    const int mi = m / T::WN, mj = m % T::WN;
                    acc[mi][mj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][mi], b[cur][mj], acc[mi][mj], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (m == 0 && kk == 0) {  // per-step loader state, needed by the loads further down
                        la.prep(k0 + 2 * kBK, k_end, lb);
                        lb.prep(k0 + 2 * kBK, k_end, la);
                    }
                    if (m == 0 && kk + 2 < kBK) {
#pragma unroll
                        for (int i = 0; i < T::WM; ++i) a[nxt][i] = As[(kk + 2 + lhi) * T::LDA + wm0 + T::WM * l32 + i];
#pragma unroll
                        for (int j = 0; j < T::WN; ++j) b[nxt][j] = Bs[(kk + 2 + lhi) * T::LDB + wn0 + j * 32 + l32];
                    }
                    if (m == 1 % NM) {
#pragma unroll
                        for (int i = 0; i < NA; ++i)
                            if (i * kGroups / NA == g) {
                                la.store(An, i, ra.r);
                                la.load(i, ra.r);
                            }
                    }
                    if (m == 2 % NM) {
#pragma unroll
                        for (int i = 0; i < NB; ++i)
                            if (i * kGroups / NB == g) {
                                lb.store(Bn, i, rb.r);
                                lb.load(i, rb.r);
                            }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __builtin_amdgcn_s_setprio(0);
            __syncthreads();
            buf ^= 1;
        }

        write_tile<T, Epi>(pe, acc, M, N, m0, n0, wm0, wn0, l32, lhi, accumulate);
        if (!tail_wg || !next_tail_item<T>(wi, tail_it, tail_end, whole_tiles, tail.ksteps, tiles_m, Kd)) break;
    }
}

// ---- the same GEMM on the bf16 matrix pipe -----------------------------------------------------
// Both operands are bf16 tensors: the tiles are kept in LDS as bf16, eight consecutive reduction
// rows of one tile position in one 16-byte cell ([BK/8][tile + pad][8]), which is exactly the
// operand of v_mfma_f32_32x32x16_bf16 for the lane that owns that position (lanes 0-31 take rows
// 0-7 of the step, lanes 32-63 rows 8-15, for A and B alike, so the products pair up whatever the
// instruction's internal order).  One MFMA per 32x32 tile covers a whole step of BK = 16 rows,
// 8 times the fp32 rate, so the loop is bound by its loads and LDS traffic rather than by the
// matrix pipe; the pipeline is the fp32 kernel's (two tiles deep, one register set, memory work
// dealt out behind the MFMAs).  The loaders hand over fp32-widened values; the LDS store writes
// their upper 16 bits back, which costs no instruction.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <class T>
struct HalfTile {
    static constexpr int kCellPad = 4;  // cells of padding per 8-row plane (shifts the planes by 16 banks)
    static constexpr int PA = T::BM + kCellPad, PB = T::BN + kCellPad;  // cells per plane
    static constexpr int A_HALFS = (kBK / 8) * PA * 8, B_HALFS = (kBK / 8) * PB * 8;
    static constexpr int HALFS = A_HALFS + B_HALFS;
};

template <class T, class ALoader, class BLoader, class Epi, class AParams, class BParams>
__global__ __launch_bounds__(kThreads) void gemm_kernel_bf16(AParams pa, BParams pb, typename Epi::Params pe,
                                                              int M, int N, int Kd, int k_chunk, int tiles_m,
                                                              int tiles_n)
{
    typedef HalfTile<T> H;
    __shared__ __attribute__((aligned(16))) uint16_t lds[2][H::HALFS];

    // bf16 outputs cannot be accumulated: no spread tail here
    const WorkItem wi = work_item<T>(Kd, k_chunk, tiles_m, tiles_n, 0);
    const int m0 = wi.m0, n0 = wi.n0, k_begin = wi.k_begin, k_end = wi.k_end;
    if constexpr (per_split<Epi>(0)) pe.out += (long)wi.split * pe.plane;

    __shared__ typename ALoader::Shared sha;
    __shared__ typename BLoader::Shared shb;
    ALoader la;
    BLoader lb;
    la.init(pa, m0, M);
    lb.init(pb, n0, N);
    la.setup(sha, k_begin, k_end, lb);
    lb.setup(shb, k_begin, k_end, la);
    if constexpr (ALoader::kHasShared || BLoader::kHasShared) __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm0 = (wave % T::WAVES_M) * (T::WM * 32);
    const int wn0 = (wave / T::WAVES_M) * (T::WN * 32);
    const int l32 = lane & 31, lhi = lane >> 5;

    f32x16 acc[T::WM][T::WN];
#pragma unroll
    for (int i = 0; i < T::WM; ++i)
#pragma unroll
        for (int j = 0; j < T::WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    typename ALoader::Regs ra;
    typename BLoader::Regs rb;
    constexpr int NA = ALoader::NE, NB = BLoader::NE, NM = T::WM * T::WN;

    // element (row, position) of a tile -> halfword index of its place in the [BK/8][P][8] layout
    auto put_a = [&](uint16_t *buf, int i) {
        const int row = la.erow(i), col = la.ecol(i);
        buf[((row >> 3) * H::PA + col) * 8 + (row & 7)] = (uint16_t)(__float_as_uint(ra.r[i]) >> 16);
    };
    auto put_b = [&](uint16_t *buf, int i) {
        const int row = lb.erow(i), col = lb.ecol(i);
        buf[H::A_HALFS + ((row >> 3) * H::PB + col) * 8 + (row & 7)] = (uint16_t)(__float_as_uint(rb.r[i]) >> 16);
    };
    // a loader whose thread owns NB consecutive rows of one position writes them as one vector
    auto put_b_cells = [&](uint16_t *buf) {
        const int row = lb.erow(0), col = lb.ecol(0);
        uint32_t *dst = reinterpret_cast<uint32_t *>(buf + H::A_HALFS + ((row >> 3) * H::PB + col) * 8 + (row & 7));
        uint32_t w[NB / 2];
#pragma unroll
        for (int i = 0; i < NB / 2; ++i)
            w[i] = (__float_as_uint(rb.r[2 * i]) >> 16) | (__float_as_uint(rb.r[2 * i + 1]) & 0xFFFF0000u);
        if constexpr (NB == 8) {
            u32x4 v = {w[0], w[1], w[2], w[3]};
            *reinterpret_cast<u32x4 *>(dst) = v;
        } else {
#pragma unroll
            for (int i = 0; i < NB / 2; ++i) dst[i] = w[i];
        }
    };

    la.prep(k_begin, k_end, lb);
    lb.prep(k_begin, k_end, la);
#pragma unroll
    for (int i = 0; i < NA; ++i) la.load(i, ra.r);
#pragma unroll
    for (int i = 0; i < NB; ++i) lb.load(i, rb.r);
#pragma unroll
    for (int i = 0; i < NA; ++i) put_a(lds[0], i);
    if constexpr (BLoader::kCellStore) {
        put_b_cells(lds[0]);
    } else {
#pragma unroll
        for (int i = 0; i < NB; ++i) put_b(lds[0], i);
    }
    la.prep(k_begin + kBK, k_end, lb);
    lb.prep(k_begin + kBK, k_end, la);
#pragma unroll
    for (int i = 0; i < NA; ++i) la.load(i, ra.r);
#pragma unroll
    for (int i = 0; i < NB; ++i) lb.load(i, rb.r);
    __syncthreads();

    int buf = 0;
    for (int k0 = k_begin; k0 < k_end; k0 += kBK) {
        if constexpr (ALoader::kHasShared || BLoader::kHasShared) {
            if (k0 != k_begin && ((k0 - k_begin) & (kTabRows - 1)) == 0) {
                __syncthreads();
                la.setup(sha, k0, k_end, lb);
                lb.setup(shb, k0, k_end, la);
                __syncthreads();
            }
        }
        const uint16_t *cur = lds[buf];
        uint16_t *nxt = lds[buf ^ 1];
        // the step's operands: one 16-byte cell per MFMA tile and lane (rows 8*lhi .. 8*lhi+7)
        bf16x8 a[T::WM], b[T::WN];
#pragma unroll
        for (int i = 0; i < T::WM; ++i)
            a[i] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const u32x4 *>(cur + (lhi * H::PA + wm0 + T::WM * l32 + i) * 8));
#pragma unroll
        for (int j = 0; j < T::WN; ++j)
            b[j] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const u32x4 *>(cur + H::A_HALFS + (lhi * H::PB + wn0 + j * 32 + l32) * 8));
        la.prep(k0 + 2 * kBK, k_end, lb);
        lb.prep(k0 + 2 * kBK, k_end, la);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const int mi = m / T::WN, mj = m % T::WN;
            acc[mi][mj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[mj], acc[mi][mj], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            // this MFMA's share of the memory work: tile s+1 registers -> LDS, then reloaded with tile s+2
#pragma unroll
            for (int i = 0; i < NA; ++i)
                if (i * NM / NA == m) {
                    put_a(nxt, i);
                    la.load(i, ra.r);
                }
            if (BLoader::kCellStore && m == 0) put_b_cells(nxt);  // all of tile s+1 at once, before any reload
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (i * NM / NB == m) {
                    if constexpr (!BLoader::kCellStore) put_b(nxt, i);
                    lb.load(i, rb.r);
                }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
        buf ^= 1;
    }

    write_tile<T, Epi>(pe, acc, M, N, m0, n0, wm0, wn0, l32, lhi, wi.accumulate);
}

// ---- bf16 kernel with vector operand loads --------------------------------------------------------
// The element-wise loaders above spend 10-24 vector instructions per bf16 MFMA (one 2-byte load, its
// address and mask arithmetic and an LDS write per element) and synchronise the workgroup every 4
// MFMAs, which is what bounds gemm_kernel_bf16.  gemm_kernel_bf16v walks the reduction in steps of
// kDeepBK = 64 rows (16 MFMAs per wave between barriers) and, where the tensors' layout allows,
// fetches several elements per load:
//   * CellKLaneT: an operand contiguous along the reduction index (the filter matrix w[k][crs] of
//     Forward): one 16-byte load is one LDS cell (8 consecutive reduction rows of one tile position).
//   * RunNLaneT: the activation gather of a stride-1 layer whose output rows are as wide as its
//     input rows (grid width == tensor width): for every tap, consecutive pixels of an image are
//     consecutive in memory, so a thread fetches 4 neighbouring pixels of one reduction row with one
//     8-byte load (2-byte aligned: the platform runs with unaligned vector memory access enabled),
//     takes 8 rows, transposes them in registers into 4 cells and writes each cell in one piece.
// Tile positions index (image, pixel) with the pixel count of an image rounded up to 4, so that a
// thread's four pixels never straddle two images; the epilogue skips the padding positions.
// An element-wise loader (BK = 16 interface) can still serve as the A operand: it is run four times
// per step.

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
constexpr int kDeepBK = 64;          // reduction rows per step of gemm_kernel_bf16v
constexpr int kDeepPlanes = kDeepBK / 8;

// LDS layout of a step's tiles: 8 planes of 8 reduction rows; a plane holds one 16-byte cell per tile
// position.  A: plane stride odd (in cells), so that the 8 cells one 128-byte global load run delivers
// (8 planes of one position, 8 lanes) fall into 8 different 4-bank groups.  B: the four cells a thread
// writes (4 neighbouring pixels) go to four sub-planes TD/4 + 2 cells apart (column n -> slot
// (n % 4) * (TD/4 + 2) + n / 4): consecutive lanes then write consecutive cells, and consecutive
// columns, as the MFMA lanes read them, still fall into different bank groups.
template <class T>
struct DeepTile {
    static constexpr int PA = T::BM + 1;
    static constexpr int SUB = T::BN / 4 + 2, PB = 4 * SUB;
    static constexpr int A_HALFS = kDeepPlanes * PA * 8, B_HALFS = kDeepPlanes * PB * 8;
    static constexpr int HALFS = A_HALFS + B_HALFS;
    static __device__ __forceinline__ int b_slot(int n) { return (n & 3) * SUB + (n >> 2); }
};

struct CellParams {
    const void *t;
    uint32_t bytes;
    int col_stride;  // elements between tile positions; reduction rows are contiguous
};

template <int TD>
struct CellKLaneT : NoSetup {
    static constexpr bool kBf16 = true;
    static constexpr bool kVecCells = true;
    static std::string name() { return "CellKLane/bf16"; }
    static constexpr int kCells = kDeepPlanes * TD;                     // cells of a step's tile
    static constexpr int NC = (kCells + kThreads - 1) / kThreads;      // per thread
    static constexpr int NE = NC;
    struct Regs { u32x4 c[NC]; };
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t voff[NC];  // byte offset of the thread's cells at reduction row 0 (kOob: no such cell)

    __device__ __forceinline__ void init(const CellParams &prm, int origin, int)
    {
        rsrc = make_rsrc_bytes(prm.t, 0, prm.bytes);
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const int id = (int)threadIdx.x + kThreads * i;
            // positions past the operand's extent read whatever lies there or zero: never stored
            // 8 consecutive threads take the 8 planes of one position: 128 contiguous bytes
            voff[i] = id < kCells ? 2u * (uint32_t)((origin + id / kDeepPlanes) * prm.col_stride + 8 * (id % kDeepPlanes)) : kOob;
        }
    }
    // rows [k0 + 8*plane, +8) of each cell's position; a cell at or past k_end reads as zero (chunks are
    // multiples of 16 rows and the reduction length a multiple of 8, so a cell is all inside or all outside)
    __device__ __forceinline__ void fetch(int k0, int k_end, Regs &r) const
    {
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const int plane = ((int)threadIdx.x + kThreads * i) % kDeepPlanes;
            const bool live = k0 + 8 * plane < k_end;
            r.c[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(live ? voff[i] : kOob), 2 * k0, 0);
        }
    }
    template <int P>
    __device__ __forceinline__ void stage(uint16_t *tile, const Regs &r) const
    {
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const int id = (int)threadIdx.x + kThreads * i;
            if (id < kCells) *reinterpret_cast<u32x4 *>(tile + ((id % kDeepPlanes) * P + id / kDeepPlanes) * 8) = r.c[i];
        }
    }
};

struct RunParams {
    const void *t;
    uint32_t bytes;
    int Ct, Ht, Wt;       // tensor channel count and plane size; the grid has Wt columns too
    int plane_px;         // pixels of the grid (its rows x Wt)
    FastDiv grid_pad;     // tile position -> (image, pixel): divisor = plane_px rounded up to 4
    FastDiv grid_w;       // pixel -> (row, column): divisor = Wt
    int add_h, add_w, dir;
    FastDiv taps, taps_w;
    int n_tap_h, n_tap_w;
    int shift_thread, shift_row;
};

// MODE 0: 1x1 unpadded layers, every element exists.  MODE 1: border masks, filters of at most 16
// taps.  MODE 2: border masks, up to 31 taps.
template <int TD, int MODE>
struct RunNLaneT : NoSetup {
    static constexpr bool MASKS = MODE != 0;
    static constexpr bool kBf16 = true;
    static constexpr bool kVecRun = true;
    static std::string name() { return std::string(MODE == 0 ? "RunNLane" : MODE == 1 ? "RunNLane<masks>" : "RunNLane<masks,taps>16>") + "/bf16"; }
    static constexpr int kGroups = TD / 4;                 // 4-pixel groups per 8-row plane
    static constexpr int kTasks = kDeepPlanes * kGroups;   // (8 rows x 4 pixels) pieces of a step's tile
    static_assert(kTasks <= kThreads, "one piece per thread");
    static constexpr int NE = 8;
    struct Regs { u32x2 d[8]; uint32_t tap[MASKS ? 8 : 1]; };
    const RunParams *p;
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t voff;       // byte offset of the thread's first pixel (shifted resource)
    uint32_t ok[MASKS ? 4 : 1];  // per pixel: bit t set = tap t inside the image
    uint32_t inside;     // bit e set = pixel e of the thread exists (is not image padding, nor past the extent)
    int grp, plane;
    bool has;
    bool edge_lo, edge_hi;  // wave-uniform: some lane's windows can reach past the tensor's start / end

    __device__ __forceinline__ void init(const RunParams &prm, int origin, int extent)
    {
        p = &prm;
        const int shift = prm.shift_thread + prm.shift_row;
        rsrc = make_rsrc_bytes(prm.t, 2l * shift, prm.bytes + 2u * (uint32_t)shift);
        const int tid = threadIdx.x;
        has = kTasks == kThreads || tid < kTasks;
        grp = tid % kGroups;
        plane = (tid / kGroups) % kDeepPlanes;
        const int j0 = origin + 4 * grp;
        uint32_t n, px;
        prm.grid_pad.divmod((uint32_t)j0, n, px);
        voff = 2u * (uint32_t)((int)n * prm.Ct * prm.Ht * prm.Wt + (int)px + prm.add_h * prm.Wt + prm.add_w +
                               prm.shift_thread);
        inside = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool exists = j0 + e < extent && (int)px + e < prm.plane_px;
            inside |= exists ? 1u << e : 0u;
            if constexpr (MASKS) {
                uint32_t okm = 0;
                if (exists) {
                    uint32_t a, b;
                    prm.grid_w.divmod(px + e, a, b);
                    const int hb = (int)a + prm.add_h, wb = (int)b + prm.add_w;
                    uint32_t okw = 0;
                    for (int q = 0; q < prm.n_tap_w; ++q)
                        if ((unsigned)(wb + prm.dir * q) < (unsigned)prm.Wt) okw |= 1u << q;
                    for (int r = 0; r < prm.n_tap_h; ++r)
                        if ((unsigned)(hb + prm.dir * r) < (unsigned)prm.Ht) okm |= okw << (r * prm.n_tap_w);
                }
                ok[e] = okm;
            }
        }
        // A thread's 4-pixel window of tap (r, s) starts (r, s) rows / columns away from its pixels: in
        // the first channel of the first image it can begin before the tensor, in the last channel of
        // the last image end behind it.  Such windows are fetched element by element (see fetch).
        const int reach = prm.n_tap_h * prm.Wt + prm.n_tap_w + 4;
        const int last_image = (int)(prm.bytes / 2u) / (prm.Ct * prm.Ht * prm.Wt) - 1;
        edge_lo = __builtin_amdgcn_ballot_w64(has && n == 0 && (int)px < reach) != 0;
        edge_hi = __builtin_amdgcn_ballot_w64(has && (int)n >= last_image && (int)px + reach > prm.Ht * prm.Wt) != 0;
    }
    // The tile of reduction rows [k0, k0 + 64): lane l decodes row k0 + l, every thread then picks up
    // its 8 rows' offsets through the LDS crossbar and issues its 8 loads.
    __device__ __forceinline__ void fetch(int k0, int k_end, Regs &r) const
    {
        const int kk = k0 + (int)(threadIdx.x & 63);
        uint32_t c, tap, tr, ts;
        p->taps.divmod((uint32_t)kk, c, tap);
        p->taps_w.divmod(tap, tr, ts);
        // rows past the end get an offset that pushes every address out of range: they read as zero
        const uint32_t so_v = kk < k_end ? 2u * (uint32_t)(((int)c * p->Ht + p->dir * (int)tr) * p->Wt +
                                                            p->dir * (int)ts + p->shift_row)
                                         : kOob;
        // rows of the first / last channel, in a wave that holds pixels near the tensor's start / end
        const int n_taps = (int)p->taps.d;
        const bool careful = (edge_lo && k0 < n_taps) || (edge_hi && k0 + kDeepBK > (p->Ct - 1) * n_taps);
        uint32_t off[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int src = 4 * (8 * plane + i);
            off[i] = voff + (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)so_v);
            if constexpr (kTasks != kThreads) off[i] = has ? off[i] : kOob;
            if constexpr (MASKS) r.tap[i] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)tap);
        }
        if (__builtin_expect(!careful, 1)) {
#pragma unroll
            for (int i = 0; i < 8; ++i) r.d[i] = __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)off[i], 0, 0);
        } else {  // only elements that exist are dereferenced (unrolled: registers cannot be indexed at run time)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint32_t h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    bool live = has && ((inside >> e) & 1u);
                    if constexpr (MASKS) live = live && ((ok[e] >> r.tap[i]) & 1u);
                    h[e] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rsrc, (int)(live ? off[i] + 2u * e : kOob), 0, 0);
                }
                r.d[i].x = h[0] | (h[1] << 16);
                r.d[i].y = h[2] | (h[3] << 16);
            }
        }
    }
    // 8 rows x 4 pixels -> 4 cells of 8 rows, border taps zeroed, each cell written in one piece into
    // sub-plane e (stride SUB cells) for pixel e
    template <int P, int SUB>
    __device__ __forceinline__ void stage(uint16_t *tile, const Regs &r) const
    {
        uint32_t lo[8], hi[8];  // pixels (0, 1) and (2, 3) of each row
        uint32_t pair01 = 0, pair23 = 0;
        constexpr bool few_taps = MODE == 1;
        if constexpr (MASKS) {
            pair01 = ok[0] | (ok[1] << 16);
            pair23 = ok[2] | (ok[3] << 16);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            lo[i] = r.d[i].x;
            hi[i] = r.d[i].y;
            if constexpr (MASKS) {
                if constexpr (few_taps) {
                    // bits `tap` of the two pixels' masks at bit 0 and bit 16; times 0xFFFF spreads each
                    // over its half of the word (no carry between the halves)
                    lo[i] &= __umul24((pair01 >> r.tap[i]) & 0x00010001u, 0xFFFFu);
                    hi[i] &= __umul24((pair23 >> r.tap[i]) & 0x00010001u, 0xFFFFu);
                } else {
                    const int k0 = __builtin_amdgcn_sbfe(ok[0], r.tap[i], 1), k1 = __builtin_amdgcn_sbfe(ok[1], r.tap[i], 1);
                    const int k2 = __builtin_amdgcn_sbfe(ok[2], r.tap[i], 1), k3 = __builtin_amdgcn_sbfe(ok[3], r.tap[i], 1);
                    lo[i] &= ((uint32_t)k0 & 0xFFFFu) | ((uint32_t)k1 & 0xFFFF0000u);
                    hi[i] &= ((uint32_t)k2 & 0xFFFFu) | ((uint32_t)k3 & 0xFFFF0000u);
                }
            }
        }
        if (!has) return;
        u32x4 c0, c1, c2, c3;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // rows 2q and 2q+1 of each pixel side by side
            c0[q] = __builtin_amdgcn_perm(lo[2 * q + 1], lo[2 * q], 0x05040100u);
            c1[q] = __builtin_amdgcn_perm(lo[2 * q + 1], lo[2 * q], 0x07060302u);
            c2[q] = __builtin_amdgcn_perm(hi[2 * q + 1], hi[2 * q], 0x05040100u);
            c3[q] = __builtin_amdgcn_perm(hi[2 * q + 1], hi[2 * q], 0x07060302u);
        }
        u32x4 *dst = reinterpret_cast<u32x4 *>(tile + (plane * P + grp) * 8);
        dst[0] = c0;
        dst[SUB] = c1;
        dst[2 * SUB] = c2;
        dst[3 * SUB] = c3;
    }
};
template <int TD> using RunNLane = RunNLaneT<TD, 0>;
template <int TD> using RunNLaneMasked = RunNLaneT<TD, 1>;
template <int TD> using RunNLaneMaskedBig = RunNLaneT<TD, 2>;

template <class L>
__host__ __device__ constexpr auto vec_cells(int) -> decltype(L::kVecCells) { return L::kVecCells; }
template <class L>
__host__ __device__ constexpr bool vec_cells(...) { return false; }
template <class L>
__host__ __device__ constexpr auto vec_run(int) -> decltype(L::kVecRun) { return L::kVecRun; }
template <class L>
__host__ __device__ constexpr bool vec_run(...) { return false; }

// B operand: RunNLaneT.  A operand: CellKLaneT, or any element-wise bf16 loader (load / erow / ecol).
// k_chunk must be a multiple of kDeepBK.
template <class T, class ALoader, class BLoader, class Epi, class AParams, class BParams>
__global__ __launch_bounds__(kThreads) void gemm_kernel_bf16v(AParams pa, BParams pb, typename Epi::Params pe,
                                                               int M, int N, int Kd, int k_chunk, int tiles_m,
                                                               int tiles_n)
{
    typedef DeepTile<T> H;
    constexpr bool kACells = vec_cells<ALoader>(0);
    constexpr int KS = kDeepBK / kBK;  // 16-row sub-steps (one MFMA per 32x32 tile each)
    __shared__ __attribute__((aligned(16))) uint16_t lds[2][H::HALFS];

    const WorkItem wi = work_item<T>(Kd, k_chunk, tiles_m, tiles_n, 0);
    const int m0 = wi.m0, n0 = wi.n0, k_begin = wi.k_begin, k_end = wi.k_end;
    if constexpr (per_split<Epi>(0)) pe.out += (long)wi.split * pe.plane;

    ALoader la;
    BLoader lb;
    la.init(pa, m0, M);
    lb.init(pb, n0, N);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm0 = (wave % T::WAVES_M) * (T::WM * 32);
    const int wn0 = (wave / T::WAVES_M) * (T::WN * 32);
    const int l32 = lane & 31, lhi = lane >> 5;

    f32x16 acc[T::WM][T::WN];
#pragma unroll
    for (int i = 0; i < T::WM; ++i)
#pragma unroll
        for (int j = 0; j < T::WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    constexpr int NA = ALoader::NE, NM = T::WM * T::WN;
    struct ElemRegs { float r[KS][kACells ? 1 : NA]; };
    typedef typename std::conditional<kACells, typename ALoader::Regs, ElemRegs>::type ARegs;
    typedef typename BLoader::Regs BRegs;
    // two register sets: global loads get two whole steps to land (a step of 16 bf16 MFMAs is far
    // shorter than the memory latency, and only two of these workgroups fit a CU)
    ARegs ra0, ra1;
    BRegs rb0, rb1;

    auto load_a = [&](int k0, ARegs &ra) {
        if constexpr (kACells) {
            la.fetch(k0, k_end, ra);
        } else {
#pragma unroll
            for (int u = 0; u < KS; ++u) {
                la.prep(k0 + u * kBK, k_end, lb);
#pragma unroll
                for (int i = 0; i < NA; ++i) la.load(i, ra.r[u]);
            }
        }
    };
    auto stage_a = [&](uint16_t *buf, const ARegs &ra) {
        if constexpr (kACells) {
            la.template stage<H::PA>(buf, ra);
        } else {
#pragma unroll
            for (int u = 0; u < KS; ++u)
#pragma unroll
                for (int i = 0; i < NA; ++i) {
                    const int row = u * kBK + la.erow(i), col = la.ecol(i);
                    buf[((row >> 3) * H::PA + col) * 8 + (row & 7)] = (uint16_t)(__float_as_uint(ra.r[u][i]) >> 16);
                }
        }
    };

    // tile 0 -> LDS; tile 1 -> set 1; tile 2 -> set 0
    load_a(k_begin, ra0);
    lb.fetch(k_begin, k_end, rb0);
    load_a(k_begin + kDeepBK, ra1);
    lb.fetch(k_begin + kDeepBK, k_end, rb1);
    stage_a(lds[0], ra0);
    lb.template stage<H::PB, H::SUB>(lds[0] + H::A_HALFS, rb0);
    load_a(k_begin + 2 * kDeepBK, ra0);
    lb.fetch(k_begin + 2 * kDeepBK, k_end, rb0);
    __syncthreads();

    // One step: MFMAs on tile s from `cur`; the register set holding tile s+1 goes to `nxt` and is
    // reloaded with tile s+3.  The memory work is dealt out behind the MFMAs.
    auto step = [&](const uint16_t *cur, uint16_t *nxt, ARegs &ra, BRegs &rb, int k0) {
        bf16x8 a[2][T::WM], b[2][T::WN];
        auto read_ops = [&](int u, int slot) {  // the operands of sub-step u: planes 2u (lanes 0-31) and 2u+1
#pragma unroll
            for (int i = 0; i < T::WM; ++i)
                a[slot][i] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const u32x4 *>(cur + ((2 * u + lhi) * H::PA + wm0 + 32 * i + l32) * 8));
#pragma unroll
            for (int j = 0; j < T::WN; ++j)
                b[slot][j] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const u32x4 *>(cur + H::A_HALFS + ((2 * u + lhi) * H::PB + H::b_slot(wn0 + j * 32 + l32)) * 8));
        };
        read_ops(0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < KS; ++u) {
            const int slot = u & 1;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int mi = m / T::WN, mj = m % T::WN;
                acc[mi][mj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[slot][mi], b[slot][mj], acc[mi][mj], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (m == 0 && u + 1 < KS) read_ops(u + 1, slot ^ 1);
                if (u == 0 && m == 1 % NM) stage_a(nxt, ra);
                if (u == 1 && m == 0) load_a(k0 + 3 * kDeepBK, ra);
                if (u == 2 && m == 0) lb.template stage<H::PB, H::SUB>(nxt + H::A_HALFS, rb);
                if (u == 3 && m == 0) lb.fetch(k0 + 3 * kDeepBK, k_end, rb);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
    };
    // steps in pairs (the two LDS buffers and register sets swap roles), an odd last one after the
    // loop: a condition between the two steps of the loop body makes the register allocator move
    // accumulators between register files in every iteration
    const int n_steps = (k_end - k_begin + kDeepBK - 1) / kDeepBK;
    int k0 = k_begin;
    for (int s = 0; s + 2 <= n_steps; s += 2, k0 += 2 * kDeepBK) {
        step(lds[0], lds[1], ra1, rb1, k0);
        step(lds[1], lds[0], ra0, rb0, k0 + kDeepBK);
    }
    if (n_steps & 1) step(lds[0], lds[1], ra1, rb1, k0);

    write_tile<T, Epi, false>(pe, acc, M, N, m0, n0, wm0, wn0, l32, lhi, false);
}

// Zero-fills the outputs of the last `tail_tiles` tiles through the epilogue's own index mapping.
template <class T, class Epi>
__global__ __launch_bounds__(kThreads) void zero_tiles_kernel(typename Epi::Params pe, int M, int N, int tiles_m,
                                                              int tiles_n, int tail_tiles)
{
    const int t = tiles_m * tiles_n - tail_tiles + (int)blockIdx.x;
    const int m0 = (t % tiles_m) * T::BM, n0 = (t / tiles_m) * T::BN;
    static_assert(kThreads % T::BN == 0, "a row of the tile per thread group");
    const int col = n0 + (int)threadIdx.x % T::BN;  // lanes along the columns: contiguous stores
    if (col >= N) return;
    Epi epi;
    if (!epi.prep(pe, col)) return;
    for (int r = threadIdx.x / T::BN; r < T::BM; r += kThreads / T::BN) {
        const int row = m0 + r;
        if (row < M) epi.store(pe, row, 0.f);
    }
}

}  // namespace ucd
