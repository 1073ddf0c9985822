"""ctypes binding of libucd.so: the same entry points as include/ucd.h, argument marshalling
only.  Device buffers are torch tensors (their ``data_ptr()``) or raw integer addresses; every
step of the convolution path runs inside the library's HIP kernels.

Loading fails loudly when the library has not been built
(``python -m paper_1804_04806_amd.build``): there is no fallback path.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libucd.so")

FWD, BWD_DATA, BWD_FILTER = 0, 1, 2
ALGO_IMPLICIT, ALGO_IM2COL, ALGO_WINOGRAD, ALGO_WINOGRAD4, ALGO_FFT, ALGO_WINOGRAD_FUSED = 0, 1, 2, 3, 4, 5
ALGO_IMPLICIT_MIRROR, ALGO_WINOGRAD5_FUSED = 6, 7
N_ALGO = 8
POLICY_UNDIVIDED, POLICY_POW2, POLICY_ALL = 0, 1, 2
TIME_INF = (1 << 64) - 1
WS_NA = (1 << 64) - 1
OK, E_INVALID, E_NULLPTR, E_UNSUPPORTED, E_WS_TOO_SMALL, E_HIP, E_NOMEM, E_INFEASIBLE = 0, -1, -2, -3, -4, -5, -6, -7

WINOGRAD_ALGOS = (ALGO_WINOGRAD, ALGO_WINOGRAD4, ALGO_WINOGRAD_FUSED, ALGO_WINOGRAD5_FUSED)
# algorithms that reach the direct result through transforms (looser rounding bound than the GEMM paths)
TRANSFORM_ALGOS = WINOGRAD_ALGOS + (ALGO_FFT,)
ALGO_NAMES = {0: "implicit", 1: "im2col", 2: "winograd", 3: "winograd4", 4: "fft", 5: "winograd-fused",
              6: "implicit-mirror", 7: "winograd5x5-fused"}
OP_NAMES = {0: "fwd", 1: "bwd_data", 2: "bwd_filter"}

EXPORTS = [
    "ucd_strerror", "ucd_version", "ucd_workspace_size", "ucd_plan_from_table", "ucd_desirable_from_table",
    "ucd_wd_solve", "ucd_plan_wd_from_tables", "ucd_plan_fixed", "ucd_plan_query", "ucd_plan_destroy",
    "ucd_plan", "ucd_plan_wd", "ucd_bench_table", "ucd_bench_clear", "ucd_conv_fwd", "ucd_conv_bwd_data",
    "ucd_conv_bwd_filter", "ucd_run_micro", "ucd_mfma_probe", "ucd_describe_micro",
    "ucd_bench_save", "ucd_bench_load", "ucd_bench_put", "ucd_plan_cached", "ucd_conv_fwd_static_ws",
    "ucd_set_deterministic",
]


class UcdError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


class LayerDesc(ctypes.Structure):
    """ucd_layer_t"""
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "dtype")]


class Micro(ctypes.Structure):
    """ucd_micro_t"""
    _fields_ = [("algo", ctypes.c_int32), ("batch", ctypes.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1804_04806_amd.build`")
        # The callers' tensors come from PyTorch, which ships a HIP runtime of its own: it has to be in the
        # process before this library's, or the library binds to the system's copy and its launches then
        # fail with "no ROCm-capable device is detected" next to a working torch.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i, u64p, szp, ip = (ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                    ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_size_t),
                                    ctypes.POINTER(ctypes.c_int))
        lp, mp, pp = ctypes.POINTER(LayerDesc), ctypes.POINTER(Micro), ctypes.POINTER(vp)
        L.ucd_strerror.restype = ctypes.c_char_p
        L.ucd_strerror.argtypes = [i]
        L.ucd_version.restype = i
        L.ucd_set_deterministic.argtypes = [i]
        L.ucd_workspace_size.restype = sz
        L.ucd_workspace_size.argtypes = [lp, i, i, i]
        L.ucd_plan_from_table.argtypes = [i, sz, i, i, u64p, szp, pp]
        L.ucd_desirable_from_table.argtypes = [i, sz, i, i, u64p, szp, u64p, szp, i, ip]
        L.ucd_wd_solve.argtypes = [i, ip, u64p, szp, sz, ip, u64p]
        L.ucd_plan_wd_from_tables.argtypes = [i, ip, i, szp, u64p, szp, sz, i, pp, szp]
        L.ucd_plan_fixed.argtypes = [lp, i, mp, i, pp]
        L.ucd_plan_query.argtypes = [vp, mp, i, ip, u64p, szp]
        L.ucd_plan_destroy.restype = None
        L.ucd_plan_destroy.argtypes = [vp]
        L.ucd_plan.argtypes = [lp, i, sz, i, vp, vp, vp, vp, vp, pp]
        L.ucd_plan_wd.argtypes = [lp, ip, i, sz, i, vp, sz, vp, sz, vp, sz, vp, vp, pp, szp]
        L.ucd_bench_table.argtypes = [lp, i, u64p, szp, i]
        L.ucd_bench_clear.restype = None
        L.ucd_conv_fwd.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.ucd_conv_fwd_static_ws.argtypes = [vp, vp, vp, vp, vp]
        L.ucd_conv_bwd_data.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.ucd_conv_bwd_filter.argtypes = [vp, vp, vp, vp, ctypes.c_float, vp, sz, vp]
        L.ucd_run_micro.argtypes = [lp, i, i, i, vp, vp, vp, ctypes.c_float, vp, sz, vp]
        L.ucd_bench_save.argtypes = [ctypes.c_char_p]
        L.ucd_bench_load.argtypes = [ctypes.c_char_p, ip]
        L.ucd_bench_put.argtypes = [lp, i, i, i, ctypes.c_uint64]
        L.ucd_plan_cached.argtypes = [lp, i, sz, i, pp]
        L.ucd_describe_micro.argtypes = [lp, i, i, i, ctypes.c_char_p, sz, ip]
        L.ucd_mfma_probe.argtypes = [i, i, i, vp, sz, vp, ctypes.POINTER(ctypes.c_double)]
        _lib = L
    return _lib


def strerror(status):
    return lib().ucd_strerror(int(status)).decode()


def _check(status, where):
    if status != OK:
        raise UcdError(status, where)


def _ptr(t):
    """Device address of a torch tensor, or an int / None passed through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def layer(shape=None, dtype=0, **kw):
    """LayerDesc from a ``synth.Shape``-like object (N,C,H,W,K,R,S,stride,pad) or keywords.
    dtype 0 = fp32 tensors; 1 = bf16 x, w, dy, y, dx with fp32 dw."""
    if shape is not None:
        return LayerDesc(shape.N, shape.C, shape.H, shape.W, shape.K, shape.R, shape.S,
                         shape.stride, shape.stride, shape.pad, shape.pad, dtype)
    d = dict(stride_h=1, stride_w=1, pad_h=0, pad_w=0, dtype=dtype)
    d.update(kw)
    return LayerDesc(**d)


class Plan:
    """Owns a ucd_plan_t*."""

    def __init__(self, handle):
        self.handle = handle

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.ucd_plan_destroy(self.handle)
            self.handle = None

    def query(self):
        """(list of (algo, batch), predicted cost in ns, workspace bytes)"""
        n = ctypes.c_int(0)
        cost = ctypes.c_uint64(0)
        ws = ctypes.c_size_t(0)
        _check(lib().ucd_plan_query(self.handle, None, 0, ctypes.byref(n), ctypes.byref(cost), ctypes.byref(ws)),
               "ucd_plan_query")
        arr = (Micro * max(n.value, 1))()
        _check(lib().ucd_plan_query(self.handle, arr, n.value, None, None, None), "ucd_plan_query")
        return [(arr[k].algo, arr[k].batch) for k in range(n.value)], cost.value, ws.value

    @property
    def micro(self):
        return self.query()[0]

    @property
    def cost_ns(self):
        return self.query()[1]

    @property
    def ws_bytes(self):
        return self.query()[2]


def ucd_version():
    return lib().ucd_version()


def ucd_set_deterministic(on):
    """Switches reproducible execution on / off (on < 0: query); returns the previous setting."""
    return lib().ucd_set_deterministic(int(on))


def ucd_workspace_size(desc, op, algo, b):
    return lib().ucd_workspace_size(ctypes.byref(desc), op, algo, b)


def _tables(B, t_ns, ws):
    n_algo = len(t_ns)
    T = (ctypes.c_uint64 * (n_algo * (B + 1)))()
    M = (ctypes.c_size_t * (n_algo * (B + 1)))()
    for a in range(n_algo):
        if len(t_ns[a]) != B + 1 or len(ws[a]) != B + 1:
            raise ValueError("tables must be [n_algo][B+1]")
        for b in range(B + 1):
            T[a * (B + 1) + b] = t_ns[a][b]
            M[a * (B + 1) + b] = ws[a][b]
    return n_algo, T, M


def ucd_plan_from_table(B, ws_limit, policy, t_ns, ws):
    n_algo, T, M = _tables(B, t_ns, ws)
    out = ctypes.c_void_p()
    _check(lib().ucd_plan_from_table(B, ws_limit, policy, n_algo, T, M, ctypes.byref(out)), "ucd_plan_from_table")
    return Plan(out)


def ucd_desirable_from_table(B, ws_limit, policy, t_ns, ws):
    """List of (time, workspace) points of C(B), by increasing workspace."""
    n_algo, T, M = _tables(B, t_ns, ws)
    n = ctypes.c_int(0)
    cap = 64
    while True:
        ft = (ctypes.c_uint64 * cap)()
        fm = (ctypes.c_size_t * cap)()
        _check(lib().ucd_desirable_from_table(B, ws_limit, policy, n_algo, T, M, ft, fm, cap, ctypes.byref(n)),
               "ucd_desirable_from_table")
        if n.value <= cap:
            return [(ft[k], fm[k]) for k in range(n.value)]
        cap = n.value


def ucd_wd_solve(fronts, budget):
    """fronts: per kernel a list of (time, workspace).  Returns (choice list, total time)."""
    nk = len(fronts)
    fn = (ctypes.c_int * nk)(*[len(f) for f in fronts])
    flat = [p for f in fronts for p in f]
    ft = (ctypes.c_uint64 * len(flat))(*[p[0] for p in flat])
    fm = (ctypes.c_size_t * len(flat))(*[p[1] for p in flat])
    choice = (ctypes.c_int * nk)()
    total = ctypes.c_uint64(0)
    _check(lib().ucd_wd_solve(nk, fn, ft, fm, budget, choice, ctypes.byref(total)), "ucd_wd_solve")
    return list(choice), total.value


def ucd_plan_wd_from_tables(Bs, tables_t, tables_ws, total_ws, policy):
    """Per-kernel tables ([n_algo][B_k+1] each).  Returns (plans, ws_offsets)."""
    nk = len(Bs)
    n_algo = len(tables_t[0])
    offs, flat_t, flat_m, o = [], [], [], 0
    for k in range(nk):
        offs.append(o)
        for a in range(n_algo):
            flat_t += list(tables_t[k][a])
            flat_m += list(tables_ws[k][a])
        o += n_algo * (Bs[k] + 1)
    Barr = (ctypes.c_int * nk)(*Bs)
    offarr = (ctypes.c_size_t * nk)(*offs)
    T = (ctypes.c_uint64 * len(flat_t))(*flat_t)
    M = (ctypes.c_size_t * len(flat_m))(*flat_m)
    plans = (ctypes.c_void_p * nk)()
    wso = (ctypes.c_size_t * nk)()
    _check(lib().ucd_plan_wd_from_tables(nk, Barr, n_algo, offarr, T, M, total_ws, policy, plans, wso),
           "ucd_plan_wd_from_tables")
    return [Plan(ctypes.c_void_p(plans[k])) for k in range(nk)], list(wso)


def ucd_plan_fixed(desc, op, micro):
    arr = (Micro * len(micro))(*[Micro(a, b) for a, b in micro])
    out = ctypes.c_void_p()
    _check(lib().ucd_plan_fixed(ctypes.byref(desc), op, arr, len(micro), ctypes.byref(out)), "ucd_plan_fixed")
    return Plan(out)


def ucd_plan(desc, op, ws_limit, policy, x, w, y, ws=None, stream=None):
    out = ctypes.c_void_p()
    _check(lib().ucd_plan(ctypes.byref(desc), op, ws_limit, policy, _ptr(x), _ptr(w), _ptr(y), _ptr(ws),
                          _stream(stream), ctypes.byref(out)), "ucd_plan")
    return Plan(out)


def ucd_plan_wd(descs, ops, total_ws, policy, x, w, y, ws=None, stream=None):
    nk = len(descs)
    Ls = (LayerDesc * nk)(*descs)
    O = (ctypes.c_int * nk)(*ops)
    plans = (ctypes.c_void_p * nk)()
    wso = (ctypes.c_size_t * nk)()
    _check(lib().ucd_plan_wd(Ls, O, nk, total_ws, policy, _ptr(x), _nbytes(x), _ptr(w), _nbytes(w), _ptr(y),
                             _nbytes(y), _ptr(ws), _stream(stream), plans, wso), "ucd_plan_wd")
    return [Plan(ctypes.c_void_p(plans[k])) for k in range(nk)], list(wso)


def ucd_bench_table(desc, op, cap_b):
    """(t_ns, ws) as lists [N_ALGO][cap_b+1] from the benchmark cache."""
    T = (ctypes.c_uint64 * (N_ALGO * (cap_b + 1)))()
    M = (ctypes.c_size_t * (N_ALGO * (cap_b + 1)))()
    _check(lib().ucd_bench_table(ctypes.byref(desc), op, T, M, cap_b), "ucd_bench_table")
    t = [[T[a * (cap_b + 1) + b] for b in range(cap_b + 1)] for a in range(N_ALGO)]
    m = [[M[a * (cap_b + 1) + b] for b in range(cap_b + 1)] for a in range(N_ALGO)]
    return t, m


def ucd_bench_clear():
    lib().ucd_bench_clear()


def ucd_conv_fwd(plan, x, w, y, ws=None, ws_bytes=None, stream=None):
    _check(lib().ucd_conv_fwd(plan.handle, _ptr(x), _ptr(w), _ptr(y), _ptr(ws),
                              _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream)), "ucd_conv_fwd")


STATIC_WS_BYTES = 64 << 20


def ucd_conv_fwd_static_ws(plan, x, w, y, stream=None):
    _check(lib().ucd_conv_fwd_static_ws(plan.handle, _ptr(x), _ptr(w), _ptr(y), _stream(stream)),
           "ucd_conv_fwd_static_ws")


def ucd_conv_bwd_data(plan, dy, w, dx, ws=None, ws_bytes=None, stream=None):
    _check(lib().ucd_conv_bwd_data(plan.handle, _ptr(dy), _ptr(w), _ptr(dx), _ptr(ws),
                                   _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream)),
           "ucd_conv_bwd_data")


def ucd_conv_bwd_filter(plan, x, dy, dw, beta=0.0, ws=None, ws_bytes=None, stream=None):
    _check(lib().ucd_conv_bwd_filter(plan.handle, _ptr(x), _ptr(dy), _ptr(dw), float(beta), _ptr(ws),
                                     _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream)),
           "ucd_conv_bwd_filter")


def ucd_run_micro(desc, op, algo, b, a, bsrc, out, beta=0.0, ws=None, ws_bytes=None, stream=None):
    _check(lib().ucd_run_micro(ctypes.byref(desc), op, algo, b, _ptr(a), _ptr(bsrc), _ptr(out), float(beta),
                               _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream)),
           "ucd_run_micro")


def ucd_mfma_probe(valu_per_mfma, blocks, iters, scratch, stream=None):
    """Enqueues the MFMA calibration loop; returns the MFMA flops one launch executes."""
    flops = ctypes.c_double(0.0)
    _check(lib().ucd_mfma_probe(valu_per_mfma, blocks, iters, _ptr(scratch), _nbytes(scratch), _stream(stream),
                                ctypes.byref(flops)), "ucd_mfma_probe")
    return flops.value


def ucd_describe_micro(desc, op, algo, b):
    """(description string, number of kernel launches) of one algorithm on one micro-batch."""
    buf = ctypes.create_string_buffer(2048)
    n = ctypes.c_int(0)
    _check(lib().ucd_describe_micro(ctypes.byref(desc), op, algo, b, buf, len(buf), ctypes.byref(n)),
           "ucd_describe_micro")
    return buf.value.decode(), n.value


def ucd_bench_save(path):
    _check(lib().ucd_bench_save(str(path).encode()), "ucd_bench_save")


def ucd_bench_load(path):
    """Merges a benchmark file into the cache; returns the number of timings read."""
    n = ctypes.c_int(0)
    _check(lib().ucd_bench_load(str(path).encode(), ctypes.byref(n)), "ucd_bench_load")
    return n.value


def ucd_bench_put(desc, op, algo, b, t_ns):
    _check(lib().ucd_bench_put(ctypes.byref(desc), op, algo, b, int(t_ns)), "ucd_bench_put")


def ucd_plan_cached(desc, op, ws_limit, policy):
    out = ctypes.c_void_p()
    _check(lib().ucd_plan_cached(ctypes.byref(desc), op, ws_limit, policy, ctypes.byref(out)), "ucd_plan_cached")
    return Plan(out)
