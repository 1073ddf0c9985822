// C-ABI of the library: validation, plan objects, the micro-batch executor, the on-device
// benchmark cache and the glue to the host planners.  See include/ucd.h for the contract
// (include/ucd_calib.h for the single-micro-batch and calibration entry points).
#include "ucd.h"
#include "ucd_calib.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <tuple>
#include <vector>

#include "kernels.h"
#include "planner.h"

using namespace ucd;

struct ucd_plan {
    bool has_layer = false;
    ucd_layer_t layer{};
    int op = 0;
    std::vector<Micro> micro;
    uint64_t cost_ns = 0;
    size_t ws_bytes = 0;
};

namespace {

constexpr int kMinTimedRuns = 2, kMaxTimedRuns = 8;
constexpr float kTimedSpanMs = 0.4f;  // reps are chosen to cover about this much device time
constexpr int kSpinUpMs = 10;         // device kept busy this long before the first timing of a call

std::atomic<int> g_deterministic{0};  // ucd_set_deterministic

bool layer_ok(const ucd_layer_t *L)
{
    if (L->N < 1 || L->C < 1 || L->H < 1 || L->W < 1 || L->K < 1 || L->R < 1 || L->S < 1) return false;
    if (L->stride_h < 1 || L->stride_w < 1 || L->pad_h < 0 || L->pad_w < 0) return false;
    if (L->H + 2 * L->pad_h < L->R || L->W + 2 * L->pad_w < L->S) return false;
    if (L->R > 31 || L->S > 31) return false;  // the gather kernels keep one validity bit per filter row / column
    if (L->dtype != 0 && L->dtype != 1) return false;
    return true;
}

Dims dims_of(const ucd_layer_t *L)
{
    Dims d;
    d.C = L->C; d.H = L->H; d.W = L->W; d.K = L->K; d.R = L->R; d.S = L->S;
    d.sh = L->stride_h; d.sw = L->stride_w; d.ph = L->pad_h; d.pw = L->pad_w;
    d.P = (L->H + 2 * L->pad_h - L->R) / L->stride_h + 1;
    d.Q = (L->W + 2 * L->pad_w - L->S) / L->stride_w + 1;
    d.dtype = L->dtype;
    d.det = g_deterministic.load() != 0;
    return d;
}

// kernels address every operand of a micro-batch through a buffer resource of at most 2 GiB
constexpr long long kMaxOperandFloats = (1ll << 29) - (1ll << 16);

bool fits_32bit(const ucd_layer_t *L, int b)
{
    const Dims d = dims_of(L);
    return (long long)b * d.C * d.H * d.W <= kMaxOperandFloats && (long long)b * d.K * d.P * d.Q <= kMaxOperandFloats &&
           (long long)d.K * d.crs() <= kMaxOperandFloats;
}

// output tile edge of a Winograd algorithm id
inline int wino_tile(int algo) { return algo == UCD_ALGO_WINOGRAD4 ? 4 : 2; }
inline bool is_winograd(int algo) { return algo == UCD_ALGO_WINOGRAD || algo == UCD_ALGO_WINOGRAD4; }
// algorithms that keep a transformed filter at the head of the workspace
inline bool keeps_filter(int algo)
{
    return is_winograd(algo) || algo == UCD_ALGO_FFT || algo == UCD_ALGO_WINOGRAD_FUSED ||
           algo == UCD_ALGO_IMPLICIT_MIRROR || algo == UCD_ALGO_WINOGRAD5_FUSED;
}

size_t ws_size(const ucd_layer_t *L, int op, int algo, int b)
{
    if (!L || !layer_ok(L) || op < 0 || op >= UCD_N_OP || b < 1 || b > L->N) return UCD_WS_NA;
    if (!fits_32bit(L, b)) return UCD_WS_NA;
    const Dims d = dims_of(L);
    // reproducible mode: BackwardFilter is the implicit GEMM's alone (its partial sums in workspace)
    if (d.det && op == UCD_BWD_FILTER && algo != UCD_ALGO_IMPLICIT) return UCD_WS_NA;
    switch (algo) {
    case UCD_ALGO_IMPLICIT:
        return d.det && op == UCD_BWD_FILTER ? implicit_det_ws_bytes(d, b) : 0;
    case UCD_ALGO_IM2COL:
        // a 1x1 stride-1 unpadded layer's column matrix is x itself: nothing to gain
        if (d.R == 1 && d.S == 1 && d.sh == 1 && d.sw == 1 && d.ph == 0 && d.pw == 0) return UCD_WS_NA;
        if ((long long)d.crs() * ((long long)b * d.P * d.Q + 4) > kMaxOperandFloats) return UCD_WS_NA;
        return im2col_ws_bytes(d, b);
    case UCD_ALGO_WINOGRAD:
    case UCD_ALGO_WINOGRAD4: {
        if (!winograd_applies(d, op)) return UCD_WS_NA;
        // every transform plane is one GEMM operand
        const int mt = wino_tile(algo), planes = (mt + 2) * (mt + 2);
        if (winograd_ws_bytes(d, op, b, mt) / (4 * planes) > (size_t)kMaxOperandFloats) return UCD_WS_NA;
        return winograd_ws_bytes(d, op, b, mt);
    }
    case UCD_ALGO_WINOGRAD_FUSED:
        if (!winograd_fused_applies(d, op)) return UCD_WS_NA;
        return op == UCD_BWD_FILTER ? winograd_fused_filter_ws_bytes(d) : winograd_fused_ws_bytes(d, op);
    case UCD_ALGO_IMPLICIT_MIRROR:
        if (!implicit_mirror_applies(d, op)) return UCD_WS_NA;
        return implicit_mirror_ws_bytes(d);
    case UCD_ALGO_WINOGRAD5_FUSED:
        if (!winograd5_applies(d, op)) return UCD_WS_NA;
        return winograd5_ws_bytes(d, op);
    case UCD_ALGO_FFT:
        if (!fft_applies(d, op)) return UCD_WS_NA;
        // every frequency plane is one GEMM operand
        if (fft_ws_bytes(d, op, b) / (4 * 144) > (size_t)kMaxOperandFloats) return UCD_WS_NA;
        return fft_ws_bytes(d, op, b);
    default:
        return UCD_WS_NA;
    }
}

// UCD_E_HIP carries no detail: with UCD_VERBOSE_ERRORS set in the environment the runtime's own text
// for the error goes to stderr
int hip_status(hipError_t e)
{
    if (e == hipSuccess) return UCD_OK;
    static const bool verbose = getenv("UCD_VERBOSE_ERRORS") != nullptr;
    if (verbose) fprintf(stderr, "ucd: HIP error %d: %s\n", (int)e, hipGetErrorString(e));
    return UCD_E_HIP;
}

// One algorithm on one micro-batch.  (a, bsrc, out) = (x, w, y) | (dy, w, dx) | (x, dy, dw).
int run_micro(const ucd_layer_t *L, int op, int algo, int b, const void *a, const void *bsrc, void *out,
              float beta, float *ws, hipStream_t s, bool filter_ready = false)
{
    const Dims d = dims_of(L);
    // tensors are read element by element (dw is always fp32); the workspace matrices with 16-byte loads
    const uintptr_t emask = d.esize() - 1, omask = op == UCD_BWD_FILTER ? 3u : emask;
    if ((((uintptr_t)a | (uintptr_t)bsrc) & emask) != 0 || ((uintptr_t)out & omask) != 0) return UCD_E_INVALID;
    if ((algo != UCD_ALGO_IMPLICIT || d.det) && ((uintptr_t)ws & 15u) != 0) return UCD_E_INVALID;
    // The launches below report failure through hipGetLastError, which also returns what an earlier,
    // unrelated call of this thread left behind (a framework probing a feature at start-up, say): drop that.
    (void)hipGetLastError();
    hipError_t e = hipErrorInvalidValue;
    switch (algo) {
    case UCD_ALGO_IMPLICIT:
        if (op == UCD_FWD) e = implicit_fwd(d, b, a, bsrc, out, s);
        else if (op == UCD_BWD_DATA) e = implicit_bwd_data(d, b, a, bsrc, out, s);
        else e = implicit_bwd_filter(d, b, a, bsrc, (float *)out, beta, ws, s);
        break;
    case UCD_ALGO_IM2COL:
        if (op == UCD_FWD) e = im2col_fwd(d, b, a, bsrc, out, ws, s);
        else if (op == UCD_BWD_DATA) e = im2col_bwd_data(d, b, a, bsrc, out, ws, s);
        else e = im2col_bwd_filter(d, b, a, bsrc, (float *)out, beta, ws, s);
        break;
    case UCD_ALGO_WINOGRAD:
    case UCD_ALGO_WINOGRAD4:
        if (op == UCD_FWD) e = winograd_fwd(d, b, a, bsrc, out, ws, filter_ready, wino_tile(algo), s);
        else if (op == UCD_BWD_DATA) e = winograd_bwd_data(d, b, a, bsrc, out, ws, filter_ready, wino_tile(algo), s);
        else e = winograd_bwd_filter(d, b, a, bsrc, (float *)out, beta, ws, wino_tile(algo), s);
        break;
    case UCD_ALGO_WINOGRAD_FUSED:
        if (op != UCD_BWD_FILTER) e = winograd_fused(d, op, b, a, bsrc, out, ws, filter_ready, s);
        else e = winograd_fused_filter(d, b, a, bsrc, (float *)out, beta, ws, s);
        break;
    case UCD_ALGO_IMPLICIT_MIRROR:
        if (op == UCD_BWD_DATA) e = implicit_bwd_data_mirror(d, b, a, bsrc, out, ws, filter_ready, s);
        break;
    case UCD_ALGO_WINOGRAD5_FUSED:
        if (op != UCD_BWD_FILTER) e = winograd5_fused(d, op, b, a, bsrc, out, ws, filter_ready, s);
        else e = winograd5_fused_filter(d, b, a, bsrc, (float *)out, beta, ws, s);
        break;
    case UCD_ALGO_FFT:
        if (op == UCD_FWD) e = fft_fwd(d, b, a, bsrc, out, ws, filter_ready, s);
        else if (op == UCD_BWD_DATA) e = fft_bwd_data(d, b, a, bsrc, out, ws, filter_ready, s);
        else e = fft_bwd_filter(d, b, a, bsrc, (float *)out, beta, ws, s);
        break;
    }
    return hip_status(e);
}

int run_plan(const ucd_plan_t *plan, int op, const void *a_, const void *bsrc_, void *out_, float beta,
             void *ws, size_t ws_bytes, void *stream)
{
    if (!plan) return UCD_E_NULLPTR;
    if (!plan->has_layer || plan->op != op) return UCD_E_INVALID;
    const char *a = (const char *)a_, *bsrc = (const char *)bsrc_;
    char *out = (char *)out_;
    if (!a || !bsrc || !out) return UCD_E_NULLPTR;
    if (plan->ws_bytes > 0 && (!ws || ws_bytes < plan->ws_bytes)) return ws ? UCD_E_WS_TOO_SMALL : UCD_E_NULLPTR;
    if (op == UCD_BWD_FILTER && beta != 0.f && beta != 1.f) return UCD_E_INVALID;
    const ucd_layer_t *L = &plan->layer;
    const Dims d = dims_of(L);
    // bytes per sample of the two activation tensors
    const size_t x_img = d.esize() * d.C * d.H * d.W, y_img = d.esize() * d.K * d.P * d.Q;
    size_t o = 0;
    bool first = true;
    int prev_algo = -1;
    for (const Micro &m : plan->micro) {
        int rc;
        // consecutive Winograd micro-batches of one call share the transformed filter in the workspace
        const bool filter_ready = keeps_filter(m.algo) && prev_algo == m.algo;
        prev_algo = m.algo;
        if (op == UCD_FWD)
            rc = run_micro(L, op, m.algo, m.batch, a + o * x_img, bsrc, out + o * y_img, 0.f, (float *)ws,
                           (hipStream_t)stream, filter_ready);
        else if (op == UCD_BWD_DATA)
            rc = run_micro(L, op, m.algo, m.batch, a + o * y_img, bsrc, out + o * x_img, 0.f, (float *)ws,
                           (hipStream_t)stream, filter_ready);
        else  // the caller's beta for the first micro-batch, output scale 1 afterwards
            rc = run_micro(L, op, m.algo, m.batch, a + o * x_img, bsrc + o * y_img, out, first ? beta : 1.f,
                           (float *)ws, (hipStream_t)stream);
        if (rc != UCD_OK) return rc;
        o += (size_t)m.batch;
        first = false;
    }
    return UCD_OK;
}

// ---- benchmark cache ------------------------------------------------------------------------
typedef std::tuple<int, int, int, int, int, int, int, int, int, int, int, int, int, int> BenchKey;
std::map<BenchKey, uint64_t> g_cache;
std::mutex g_cache_mu;

BenchKey key_of(const ucd_layer_t *L, int op, int algo, int b)
{
    // timings of the reproducible mode are kept apart (dtype field + 16)
    return BenchKey(L->C, L->H, L->W, L->K, L->R, L->S, L->stride_h, L->stride_w, L->pad_h, L->pad_w,
                    L->dtype + (g_deterministic.load() != 0 ? 16 : 0), op, algo, b);
}

bool cache_get(const BenchKey &k, uint64_t &t)
{
    std::lock_guard<std::mutex> g(g_cache_mu);
    auto it = g_cache.find(k);
    if (it == g_cache.end()) return false;
    t = it->second;
    return true;
}

void cache_put(const BenchKey &k, uint64_t t)
{
    std::lock_guard<std::mutex> g(g_cache_mu);
    g_cache[k] = t;
}

struct Events {
    hipEvent_t a = nullptr, b = nullptr;
    ~Events()
    {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

// Device time of one (algo, b) as it will cost inside a configuration: after one warm-up run, a
// few runs are launched back to back on consecutive micro-batches of the buffers (wrapping at N),
// and the time per run between two events around the whole sequence is taken, in integer ns.
// Timed like this a run includes the dispatch gap to its successor, reads activations that the
// previous run has not just pulled into the caches, and sees the clock of a busy chip: the three
// things a lone, repeated run on the same samples leaves out, all of which favour small
// micro-batches and made configurations look faster than they then ran.
int time_micro(const ucd_layer_t *L, int op, int algo, int b, void *x, void *w, void *y, float *ws,
               hipStream_t s, Events &ev, uint64_t &ns)
{
    const Dims d = dims_of(L);
    const size_t x_img = d.esize() * d.C * d.H * d.W, y_img = d.esize() * d.K * d.P * d.Q;
    // BackwardFilter is timed as the accumulating call it is for every micro-batch but the first
    const float beta = op == UCD_BWD_FILTER ? 1.f : 0.f;
    if (op == UCD_BWD_FILTER && fill_zero((float *)w, (size_t)d.K * d.crs(), s) != hipSuccess) return UCD_E_HIP;
    auto run_at = [&](int o, bool filter_ready) {  // the micro-batch of samples o .. o+b-1
        char *xo = (char *)x + (size_t)o * x_img, *yo = (char *)y + (size_t)o * y_img;
        if (op == UCD_FWD) return run_micro(L, op, algo, b, xo, w, yo, beta, ws, s, filter_ready);
        if (op == UCD_BWD_DATA) return run_micro(L, op, algo, b, yo, w, xo, beta, ws, s, filter_ready);
        return run_micro(L, op, algo, b, xo, yo, w, beta, ws, s);
    };
    // A configuration holds at most N / b micro-batches of this size, and the executor transforms
    // the filter once per run of one algorithm: the timed sequence does the same, so that a
    // transforming algorithm's entry carries the share of the filter transform it will really pay.
    const int per_config = std::max(1, L->N / b);
    auto elapsed = [&](float &ms) {
        if (hipEventRecord(ev.b, s) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess) return UCD_E_HIP;
        return hipEventElapsedTime(&ms, ev.a, ev.b) == hipSuccess ? UCD_OK : UCD_E_HIP;
    };
    float warm = 0.f, total = 0.f;
    if (hipEventRecord(ev.a, s) != hipSuccess) return UCD_E_HIP;
    int rc = run_at(0, false);
    if (rc != UCD_OK || (rc = elapsed(warm)) != UCD_OK) return rc;
    int reps = warm > 0.f ? (int)(kTimedSpanMs / warm) : kMaxTimedRuns;
    reps = reps < kMinTimedRuns ? kMinTimedRuns : (reps > kMaxTimedRuns ? kMaxTimedRuns : reps);
    if (hipEventRecord(ev.a, s) != hipSuccess) return UCD_E_HIP;
    for (int it = 0, o = 0; it < reps; ++it) {
        o = o + 2 * b <= L->N ? o + b : 0;  // the next micro-batch, starting after the warm-up's
        if ((rc = run_at(o, keeps_filter(algo) && it % per_config != 0)) != UCD_OK) return rc;
    }
    if ((rc = elapsed(total)) != UCD_OK) return rc;
    ns = (uint64_t)std::llround((double)total / reps * 1e6);
    if (ns == 0) ns = 1;
    return UCD_OK;
}

// Step 1 of the WR algorithm for one kernel: fill the table for every policy size and every
// algorithm that applies and fits `limit`, timing what the cache does not hold yet.
int bench_kernel(const ucd_layer_t *L, int op, size_t limit, int policy, void *x, void *w, void *y, float *ws,
                 hipStream_t s, std::vector<uint64_t> &t, std::vector<size_t> &m)
{
    const int B = L->N;
    t.assign((size_t)UCD_N_ALGO * (B + 1), kTimeInf);
    m.assign((size_t)UCD_N_ALGO * (B + 1), kWsNa);
    Events ev;
    if (hipEventCreate(&ev.a) != hipSuccess || hipEventCreate(&ev.b) != hipSuccess) return UCD_E_HIP;
    bool spun = false;
    for (int b : policy_sizes(policy, B))
        for (int a = 0; a < UCD_N_ALGO; ++a) {
            const size_t need = ws_size(L, op, a, b);
            if (need == UCD_WS_NA) continue;
            m[(size_t)a * (B + 1) + b] = need;
            if (need > limit) continue;
            const BenchKey k = key_of(L, op, a, b);
            uint64_t ns;
            if (!cache_get(k, ns)) {
                if (!spun) {
                    // A GPU that has sat idle (while the host prepared tensors, say) runs its first
                    // kernels at a low clock: timings taken then came out 5-15 % too long, and since
                    // they are cached, later plans compared fresh timings against stale slow ones.
                    // Keep the device busy for a few milliseconds before the first measurement.
                    const auto t0 = std::chrono::steady_clock::now();
                    do {
                        int rc = time_micro(L, op, a, b, x, w, y, ws, s, ev, ns);
                        if (rc != UCD_OK) return rc;
                    } while (std::chrono::steady_clock::now() - t0 < std::chrono::milliseconds(kSpinUpMs));
                    spun = true;
                }
                int rc = time_micro(L, op, a, b, x, w, y, ws, s, ev, ns);
                if (rc != UCD_OK) return rc;
                cache_put(k, ns);
            }
            t[(size_t)a * (B + 1) + b] = ns;
        }
    return UCD_OK;
}

// group = true: a planner's configuration, whose micro-batches may run in any order, is stored with
// those of one algorithm next to each other, so that consecutive Winograd micro-batches share
// the transformed filter (see run_plan).  A caller's fixed configuration keeps its order.
ucd_plan_t *make_plan(const Config &cfg, const ucd_layer_t *L, int op, bool group = true)
{
    ucd_plan_t *p = new (std::nothrow) ucd_plan_t();
    if (!p) return nullptr;
    p->micro = cfg.micro;
    if (group)
        std::stable_sort(p->micro.begin(), p->micro.end(), [](const Micro &a, const Micro &b) { return a.algo < b.algo; });
    p->cost_ns = cfg.cost;
    p->ws_bytes = cfg.ws;
    p->op = op;
    if (L) {
        p->has_layer = true;
        p->layer = *L;
    }
    return p;
}

bool policy_ok(int policy) { return policy >= UCD_POLICY_UNDIVIDED && policy <= UCD_POLICY_ALL; }

size_t round256(size_t v) { return (v + 255) / 256 * 256; }

// Desirable sets -> 0-1 programme -> per-kernel configurations and segment offsets.
int solve_wd(const std::vector<std::vector<Config>> &fronts, size_t total_ws, std::vector<int> &choice)
{
    std::vector<std::vector<FrontPoint>> pts(fronts.size());
    for (size_t k = 0; k < fronts.size(); ++k)
        for (const Config &c : fronts[k]) pts[k].push_back({c.cost, round256(c.ws)});
    uint64_t total;
    if (!wd_solve(pts, total_ws, choice, total)) return UCD_E_INFEASIBLE;
    return UCD_OK;
}

// ---- workspace held by the library, for callers that cannot allocate ------------------------------
// One array per GPU, in the code object's zero-initialised data: it exists from module load to
// process end.  The name below is only the host-side handle of the symbol; its device address is
// looked up once per device with that device current, and only that address is ever handed to a launch.
constexpr size_t kStaticWsBytes = UCD_STATIC_WS_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

int static_workspace(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return UCD_E_HIP;
    if (dev < 0 || dev >= kMaxDevices) return UCD_E_UNSUPPORTED;
    std::lock_guard<std::mutex> g(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return UCD_E_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return UCD_OK;
}

// No C++ exception may cross the C boundary: allocation failures become UCD_E_NOMEM.
template <class F>
int guarded(F body) noexcept
{
    try {
        return body();
    } catch (const std::bad_alloc &) {
        return UCD_E_NOMEM;
    } catch (...) {
        return UCD_E_INVALID;
    }
}

}  // namespace

// ---- exported ------------------------------------------------------------------------------
extern "C" {

const char *ucd_strerror(int status)
{
    switch (status) {
    case UCD_OK: return "ok";
    case UCD_E_INVALID: return "invalid argument";
    case UCD_E_NULLPTR: return "null pointer";
    case UCD_E_UNSUPPORTED: return "algorithm or dtype not supported for this layer";
    case UCD_E_WS_TOO_SMALL: return "workspace smaller than the plan needs";
    case UCD_E_HIP: return "HIP runtime error";
    case UCD_E_NOMEM: return "out of host memory";
    case UCD_E_INFEASIBLE: return "no feasible configuration";
    default: return "unknown status";
    }
}

int ucd_version(void) { return 101; }

int ucd_set_deterministic(int on)
{
    if (on < 0) return g_deterministic.load();
    return g_deterministic.exchange(on != 0 ? 1 : 0);
}

size_t ucd_workspace_size(const ucd_layer_t *layer, int op, int algo, int b) { return ws_size(layer, op, algo, b); }

int ucd_plan_from_table(int B, size_t ws_limit, int policy, int n_algo, const uint64_t *t_ns, const size_t *ws,
                        ucd_plan_t **out)
{
    return guarded([&]() -> int {
        if (!t_ns || !ws || !out) return UCD_E_NULLPTR;
        if (B < 1 || n_algo < 1 || !policy_ok(policy)) return UCD_E_INVALID;
        Table tab{B, n_algo, t_ns, ws};
        Config cfg;
        if (!wr_plan(tab, ws_limit, policy, cfg)) return UCD_E_INFEASIBLE;
        ucd_plan_t *p = make_plan(cfg, nullptr, 0);
        if (!p) return UCD_E_NOMEM;
        *out = p;
        return UCD_OK;
    });
}

int ucd_desirable_from_table(int B, size_t ws_limit, int policy, int n_algo, const uint64_t *t_ns,
                             const size_t *ws, uint64_t *front_t, size_t *front_ws, int cap, int *n)
{
    return guarded([&]() -> int {
        if (!t_ns || !ws || !n || (cap > 0 && (!front_t || !front_ws))) return UCD_E_NULLPTR;
        if (B < 1 || n_algo < 1 || !policy_ok(policy) || cap < 0) return UCD_E_INVALID;
        Table tab{B, n_algo, t_ns, ws};
        std::vector<Config> front;
        if (!desirable_set(tab, ws_limit, policy, front)) return UCD_E_INFEASIBLE;
        for (int i = 0; i < (int)front.size() && i < cap; ++i) {
            front_t[i] = front[i].cost;
            front_ws[i] = front[i].ws;
        }
        *n = (int)front.size();
        return UCD_OK;
    });
}

int ucd_wd_solve(int n_kernels, const int *front_n, const uint64_t *front_t, const size_t *front_ws,
                 size_t budget, int *choice, uint64_t *total_t)
{
    return guarded([&]() -> int {
        if (!front_n || !front_t || !front_ws || !choice || !total_t) return UCD_E_NULLPTR;
        if (n_kernels < 1) return UCD_E_INVALID;
        std::vector<std::vector<FrontPoint>> pts(n_kernels);
        size_t o = 0;
        for (int k = 0; k < n_kernels; ++k) {
            if (front_n[k] < 1) return UCD_E_INVALID;
            for (int i = 0; i < front_n[k]; ++i, ++o) pts[k].push_back({front_t[o], front_ws[o]});
        }
        std::vector<int> ch;
        uint64_t total;
        if (!wd_solve(pts, budget, ch, total)) return UCD_E_INFEASIBLE;
        std::copy(ch.begin(), ch.end(), choice);
        *total_t = total;
        return UCD_OK;
    });
}

int ucd_plan_wd_from_tables(int n_kernels, const int *B, int n_algo, const size_t *tab_off, const uint64_t *t_ns,
                            const size_t *ws, size_t total_ws, int policy, ucd_plan_t **plans, size_t *ws_offsets)
{
    return guarded([&]() -> int {
        if (!B || !tab_off || !t_ns || !ws || !plans || !ws_offsets) return UCD_E_NULLPTR;
        if (n_kernels < 1 || n_algo < 1 || !policy_ok(policy)) return UCD_E_INVALID;
        std::vector<std::vector<Config>> fronts(n_kernels);
        for (int k = 0; k < n_kernels; ++k) {
            if (B[k] < 1) return UCD_E_INVALID;
            Table tab{B[k], n_algo, t_ns + tab_off[k], ws + tab_off[k]};
            if (!desirable_set(tab, total_ws, policy, fronts[k])) return UCD_E_INFEASIBLE;
        }
        std::vector<int> choice;
        int rc = solve_wd(fronts, total_ws, choice);
        if (rc != UCD_OK) return rc;
        std::vector<ucd_plan_t *> made;
        for (int k = 0; k < n_kernels; ++k) {
            ucd_plan_t *p = make_plan(fronts[k][choice[k]], nullptr, 0);
            if (!p) {
                for (ucd_plan_t *q : made) delete q;
                return UCD_E_NOMEM;
            }
            made.push_back(p);
        }
        size_t off = 0;
        for (int k = 0; k < n_kernels; ++k) {
            plans[k] = made[k];
            ws_offsets[k] = off;
            off += round256(made[k]->ws_bytes);
        }
        return UCD_OK;
    });
}

int ucd_plan_fixed(const ucd_layer_t *layer, int op, const ucd_micro_t *micro, int n, ucd_plan_t **out)
{
    return guarded([&]() -> int {
        if (!layer || !micro || !out) return UCD_E_NULLPTR;
        if (!layer_ok(layer) || op < 0 || op >= UCD_N_OP || n < 1) return UCD_E_INVALID;
        Config cfg;
        long sum = 0;
        for (int i = 0; i < n; ++i) {
            if (micro[i].batch < 1 || micro[i].batch > layer->N) return UCD_E_INVALID;
            if (micro[i].algo < 0 || micro[i].algo >= UCD_N_ALGO) return UCD_E_INVALID;
            const size_t need = ws_size(layer, op, micro[i].algo, micro[i].batch);
            if (need == UCD_WS_NA) return UCD_E_UNSUPPORTED;
            cfg.ws = std::max(cfg.ws, need);
            cfg.micro.push_back({micro[i].algo, micro[i].batch});
            sum += micro[i].batch;
        }
        if (sum != layer->N) return UCD_E_INVALID;
        ucd_plan_t *p = make_plan(cfg, layer, op, false);
        if (!p) return UCD_E_NOMEM;
        *out = p;
        return UCD_OK;
    });
}

int ucd_plan_query(const ucd_plan_t *plan, ucd_micro_t *micro, int cap, int *n, uint64_t *cost_ns, size_t *ws_bytes)
{
    return guarded([&]() -> int {
        if (!plan) return UCD_E_NULLPTR;
        if (cap < 0 || (cap > 0 && !micro)) return UCD_E_INVALID;
        for (int i = 0; i < cap && i < (int)plan->micro.size(); ++i) {
            micro[i].algo = plan->micro[i].algo;
            micro[i].batch = plan->micro[i].batch;
        }
        if (n) *n = (int)plan->micro.size();
        if (cost_ns) *cost_ns = plan->cost_ns;
        if (ws_bytes) *ws_bytes = plan->ws_bytes;
        return UCD_OK;
    });
}

void ucd_plan_destroy(ucd_plan_t *plan) { delete plan; }

int ucd_plan(const ucd_layer_t *layer, int op, size_t ws_limit, int policy, void *x, void *w, void *y, void *ws,
             void *stream, ucd_plan_t **out)
{
    return guarded([&]() -> int {
        if (!layer || !x || !w || !y || !out) return UCD_E_NULLPTR;
        if (!layer_ok(layer) || op < 0 || op >= UCD_N_OP || !policy_ok(policy)) return UCD_E_INVALID;
        if (!fits_32bit(layer, layer->N)) return UCD_E_UNSUPPORTED;
        if (ws_limit > 0 && !ws) return UCD_E_NULLPTR;
        std::vector<uint64_t> t;
        std::vector<size_t> m;
        int rc = bench_kernel(layer, op, ws_limit, policy, x, w, y, (float *)ws,
                              (hipStream_t)stream, t, m);
        if (rc != UCD_OK) return rc;
        Table tab{layer->N, UCD_N_ALGO, t.data(), m.data()};
        Config cfg;
        if (!wr_plan(tab, ws_limit, policy, cfg)) return UCD_E_INFEASIBLE;
        ucd_plan_t *p = make_plan(cfg, layer, op);
        if (!p) return UCD_E_NOMEM;
        *out = p;
        return UCD_OK;
    });
}

int ucd_plan_wd(const ucd_layer_t *layers, const int *ops, int n_kernels, size_t total_ws, int policy, void *x,
                size_t x_cap, void *w, size_t w_cap, void *y, size_t y_cap, void *ws, void *stream,
                ucd_plan_t **plans, size_t *ws_offsets)
{
    return guarded([&]() -> int {
        if (!layers || !ops || !x || !w || !y || !plans || !ws_offsets) return UCD_E_NULLPTR;
        if (n_kernels < 1 || !policy_ok(policy)) return UCD_E_INVALID;
        if (total_ws > 0 && !ws) return UCD_E_NULLPTR;
        for (int k = 0; k < n_kernels; ++k) {
            const ucd_layer_t *L = &layers[k];
            if (!layer_ok(L) || ops[k] < 0 || ops[k] >= UCD_N_OP) return UCD_E_INVALID;
            if (!fits_32bit(L, L->N)) return UCD_E_UNSUPPORTED;
            const Dims d = dims_of(L);
            // the w scratch doubles as the fp32 dw of BackwardFilter kernels
            if ((size_t)L->N * d.C * d.H * d.W * d.esize() > x_cap || (size_t)d.K * d.crs() * 4 > w_cap ||
                (size_t)L->N * d.K * d.P * d.Q * d.esize() > y_cap)
                return UCD_E_INVALID;
        }
        std::vector<std::vector<Config>> fronts(n_kernels);
        for (int k = 0; k < n_kernels; ++k) {
            std::vector<uint64_t> t;
            std::vector<size_t> m;
            int rc = bench_kernel(&layers[k], ops[k], total_ws, policy, x, w, y, (float *)ws,
                                  (hipStream_t)stream, t, m);
            if (rc != UCD_OK) return rc;
            Table tab{layers[k].N, UCD_N_ALGO, t.data(), m.data()};
            if (!desirable_set(tab, total_ws, policy, fronts[k])) return UCD_E_INFEASIBLE;
        }
        std::vector<int> choice;
        int rc = solve_wd(fronts, total_ws, choice);
        if (rc != UCD_OK) return rc;
        std::vector<ucd_plan_t *> made;
        for (int k = 0; k < n_kernels; ++k) {
            ucd_plan_t *p = make_plan(fronts[k][choice[k]], &layers[k], ops[k]);
            if (!p) {
                for (ucd_plan_t *q : made) delete q;
                return UCD_E_NOMEM;
            }
            made.push_back(p);
        }
        size_t off = 0;
        for (int k = 0; k < n_kernels; ++k) {
            plans[k] = made[k];
            ws_offsets[k] = off;
            off += round256(made[k]->ws_bytes);
        }
        return UCD_OK;
    });
}

int ucd_bench_table(const ucd_layer_t *layer, int op, uint64_t *t_ns, size_t *ws, int cap_b)
{
    return guarded([&]() -> int {
        if (!layer || !t_ns || !ws) return UCD_E_NULLPTR;
        if (!layer_ok(layer) || op < 0 || op >= UCD_N_OP || cap_b < 1) return UCD_E_INVALID;
        ucd_layer_t L = *layer;
        for (int a = 0; a < UCD_N_ALGO; ++a)
            for (int b = 0; b <= cap_b; ++b) {
                const size_t i = (size_t)a * (cap_b + 1) + b;
                t_ns[i] = UCD_TIME_INF;
                ws[i] = UCD_WS_NA;
                if (b < 1) continue;
                L.N = std::max(L.N, b);
                ws[i] = ws_size(&L, op, a, b);
                uint64_t ns;
                if (cache_get(key_of(&L, op, a, b), ns)) t_ns[i] = ns;
            }
        return UCD_OK;
    });
}

void ucd_bench_clear(void)
{
    std::lock_guard<std::mutex> g(g_cache_mu);
    g_cache.clear();
}

int ucd_bench_put(const ucd_layer_t *layer, int op, int algo, int b, uint64_t t_ns)
{
    return guarded([&]() -> int {
        if (!layer) return UCD_E_NULLPTR;
        if (!layer_ok(layer) || op < 0 || op >= UCD_N_OP || algo < 0 || algo >= UCD_N_ALGO || b < 1 || t_ns == 0 ||
            t_ns == UCD_TIME_INF)
            return UCD_E_INVALID;
        cache_put(key_of(layer, op, algo, b), t_ns);
        return UCD_OK;
    });
}

// File format: one header line "ucd-bench 1 <device>", then one line of 15 integers per timing:
// C H W K R S stride_h stride_w pad_h pad_w dtype op algo b ns.
static std::string device_tag()
{
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        return "none";
    }
    std::string tag = std::string(prop.gcnArchName) + "/" + std::to_string(prop.multiProcessorCount) + "cu";
    for (char &ch : tag)
        if (ch == ' ') ch = '_';
    return tag;
}

int ucd_bench_save(const char *path)
{
    return guarded([&]() -> int {
        if (!path) return UCD_E_NULLPTR;
        FILE *f = std::fopen(path, "w");
        if (!f) return UCD_E_INVALID;
        std::fprintf(f, "ucd-bench 1 %s\n", device_tag().c_str());
        std::lock_guard<std::mutex> g(g_cache_mu);
        for (const auto &kv : g_cache) {
            const BenchKey &k = kv.first;
            std::fprintf(f, "%d %d %d %d %d %d %d %d %d %d %d %d %d %d %llu\n", std::get<0>(k), std::get<1>(k),
                         std::get<2>(k), std::get<3>(k), std::get<4>(k), std::get<5>(k), std::get<6>(k), std::get<7>(k),
                         std::get<8>(k), std::get<9>(k), std::get<10>(k), std::get<11>(k), std::get<12>(k), std::get<13>(k),
                         (unsigned long long)kv.second);
        }
        const bool ok = std::fclose(f) == 0;
        return ok ? UCD_OK : UCD_E_INVALID;
    });
}

int ucd_bench_load(const char *path, int *n_loaded)
{
    return guarded([&]() -> int {
        if (!path) return UCD_E_NULLPTR;
        FILE *f = std::fopen(path, "r");
        if (!f) return UCD_E_INVALID;
        char magic[32] = {0}, dev[128] = {0};
        int ver = 0;
        if (std::fscanf(f, "%31s %d %127s", magic, &ver, dev) != 3 || std::strcmp(magic, "ucd-bench") != 0 || ver != 1) {
            std::fclose(f);
            return UCD_E_INVALID;
        }
        // timings are only meaningful on the device they were taken on; a process without a GPU
        // (offline planning) accepts any file
        const std::string here = device_tag();
        if (here != "none" && std::strcmp(dev, "none") != 0 && here != dev) {
            std::fclose(f);
            return UCD_E_UNSUPPORTED;
        }
        std::vector<std::pair<BenchKey, uint64_t>> rows;
        int v[14];
        unsigned long long ns;
        for (;;) {
            int got = 0;
            for (int i = 0; i < 14; ++i) got += std::fscanf(f, "%d", &v[i]) == 1;
            if (got == 0) break;
            if (got != 14 || std::fscanf(f, "%llu", &ns) != 1 || ns == 0) {
                std::fclose(f);
                return UCD_E_INVALID;
            }
            rows.push_back({BenchKey(v[0], v[1], v[2], v[3], v[4], v[5], v[6], v[7], v[8], v[9], v[10], v[11], v[12], v[13]),
                            (uint64_t)ns});
        }
        std::fclose(f);
        for (const auto &r : rows) cache_put(r.first, r.second);
        if (n_loaded) *n_loaded = (int)rows.size();
        return UCD_OK;
    });
}

int ucd_plan_cached(const ucd_layer_t *layer, int op, size_t ws_limit, int policy, ucd_plan_t **out)
{
    return guarded([&]() -> int {
        if (!layer || !out) return UCD_E_NULLPTR;
        if (!layer_ok(layer) || op < 0 || op >= UCD_N_OP || !policy_ok(policy)) return UCD_E_INVALID;
        if (!fits_32bit(layer, layer->N)) return UCD_E_UNSUPPORTED;
        const int B = layer->N;
        std::vector<uint64_t> t((size_t)UCD_N_ALGO * (B + 1), kTimeInf);
        std::vector<size_t> m((size_t)UCD_N_ALGO * (B + 1), kWsNa);
        for (int b : policy_sizes(policy, B))
            for (int a = 0; a < UCD_N_ALGO; ++a) {
                const size_t need = ws_size(layer, op, a, b);
                if (need == UCD_WS_NA) continue;
                m[(size_t)a * (B + 1) + b] = need;
                uint64_t ns;
                if (need <= ws_limit && cache_get(key_of(layer, op, a, b), ns)) t[(size_t)a * (B + 1) + b] = ns;
            }
        Table tab{B, UCD_N_ALGO, t.data(), m.data()};
        Config cfg;
        if (!wr_plan(tab, ws_limit, policy, cfg)) return UCD_E_INFEASIBLE;
        ucd_plan_t *p = make_plan(cfg, layer, op);
        if (!p) return UCD_E_NOMEM;
        *out = p;
        return UCD_OK;
    });
}

int ucd_conv_fwd(const ucd_plan_t *plan, const void *x, const void *w, void *y, void *ws, size_t ws_bytes,
                 void *stream)
{
    return guarded([&]() -> int {
        return run_plan(plan, UCD_FWD, x, w, y, 0.f, ws, ws_bytes, stream);
    });
}

int ucd_conv_fwd_static_ws(const ucd_plan_t *plan, const void *x, const void *w, void *y, void *stream)
{
    return guarded([&]() -> int {
        if (!plan) return UCD_E_NULLPTR;
        if (plan->ws_bytes > kStaticWsBytes) return UCD_E_WS_TOO_SMALL;
        void *ws = nullptr;
        if (plan->ws_bytes > 0) {
            const int rc = static_workspace(&ws);
            if (rc != UCD_OK) return rc;
        }
        return run_plan(plan, UCD_FWD, x, w, y, 0.f, ws, kStaticWsBytes, stream);
    });
}

int ucd_conv_bwd_data(const ucd_plan_t *plan, const void *dy, const void *w, void *dx, void *ws, size_t ws_bytes,
                      void *stream)
{
    return guarded([&]() -> int {
        return run_plan(plan, UCD_BWD_DATA, dy, w, dx, 0.f, ws, ws_bytes, stream);
    });
}

int ucd_conv_bwd_filter(const ucd_plan_t *plan, const void *x, const void *dy, void *dw, float beta, void *ws,
                        size_t ws_bytes, void *stream)
{
    return guarded([&]() -> int {
        return run_plan(plan, UCD_BWD_FILTER, x, dy, dw, beta, ws, ws_bytes,
                        stream);
    });
}

int ucd_describe_micro(const ucd_layer_t *layer, int op, int algo, int b, char *buf, size_t cap, int *n_launches)
{
    return guarded([&]() -> int {
        if (!layer || !buf) return UCD_E_NULLPTR;
        if (!layer_ok(layer) || op < 0 || op >= UCD_N_OP || b < 1 || cap < 1) return UCD_E_INVALID;
        ucd_layer_t L = *layer;
        L.N = std::max(L.N, b);
        if (ws_size(&L, op, algo, b) == UCD_WS_NA) return UCD_E_UNSUPPORTED;
        LaunchLog log;
        launch_log() = &log;
        // pointers are only passed through to the (suppressed) launches, never dereferenced on the host
        int rc = run_micro(&L, op, algo, b, nullptr, nullptr, nullptr, op == UCD_BWD_FILTER ? 1.f : 0.f, nullptr, nullptr);
        launch_log() = nullptr;
        if (rc != UCD_OK) return rc;
        const size_t n = std::min(cap - 1, log.text.size());
        std::memcpy(buf, log.text.data(), n);
        buf[n] = 0;
        if (n_launches) *n_launches = log.launches;
        return UCD_OK;
    });
}

int ucd_mfma_probe(int valu_per_mfma, int blocks, int iters, void *scratch, size_t scratch_bytes, void *stream,
                   double *flops)
{
    return guarded([&]() -> int {
        if (!scratch || !flops) return UCD_E_NULLPTR;
        if (blocks < 1 || blocks > 65536 || iters < 1 || scratch_bytes < (size_t)blocks * 256 * 4) return UCD_E_INVALID;
        hipError_t e = mfma_probe(valu_per_mfma, blocks, iters, (float *)scratch, (hipStream_t)stream);
        if (e == hipErrorInvalidValue) return UCD_E_INVALID;
        if (e != hipSuccess) return UCD_E_HIP;
        *flops = (double)blocks * 4.0 * iters * 16.0 * 4096.0;
        return UCD_OK;
    });
}

int ucd_run_micro(const ucd_layer_t *layer, int op, int algo, int b, const void *a, const void *bsrc, void *out,
                  float beta, void *ws, size_t ws_bytes, void *stream)
{
    return guarded([&]() -> int {
        if (!layer || !a || !bsrc || !out) return UCD_E_NULLPTR;
        // the descriptor's N is the extent of the caller's buffers: a micro-batch cannot exceed it
        if (!layer_ok(layer) || op < 0 || op >= UCD_N_OP || b < 1 || b > layer->N) return UCD_E_INVALID;
        ucd_layer_t L = *layer;
        const size_t need = ws_size(&L, op, algo, b);
        if (need == UCD_WS_NA) return UCD_E_UNSUPPORTED;
        if (need > 0 && !ws) return UCD_E_NULLPTR;
        if (need > ws_bytes) return UCD_E_WS_TOO_SMALL;
        if (op == UCD_BWD_FILTER && beta != 0.f && beta != 1.f) return UCD_E_INVALID;
        return run_micro(&L, op, algo, b, a, bsrc, out, beta, (float *)ws,
                         (hipStream_t)stream);
    });
}

}  // extern "C"
