"""The C-ABI library loads without a GPU and exports every symbol include/*.h declares."""
import ctypes
import os
import re

from paper_1804_04806_amd import ucd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("ucd.h", "ucd_calib.h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ucd_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_symbols()
    assert len(names) >= 18 and "ucd_plan" in names and "ucd_conv_bwd_filter" in names
    lib = ctypes.CDLL(ucd.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(ucd.EXPORTS) == names


def test_version_and_strerror():
    assert ucd.ucd_version() >= 100
    assert ucd.strerror(0) == "ok" and "workspace" in ucd.strerror(ucd.E_WS_TOO_SMALL)


def test_workspace_formulas():
    L = ucd.layer(N=8, C=16, H=16, W=16, K=32, R=3, S=3, pad_h=1, pad_w=1)
    assert ucd.ucd_workspace_size(L, ucd.FWD, ucd.ALGO_IMPLICIT, 8) == 0
    # im2col: 4 bytes x C*R*S x (b*P*Q rounded up to 4): 144 KiB per image here
    assert ucd.ucd_workspace_size(L, ucd.FWD, ucd.ALGO_IM2COL, 1) == 4 * 144 * 256 == 147456
    assert ucd.ucd_workspace_size(L, ucd.BWD_FILTER, ucd.ALGO_IM2COL, 3) == 3 * 147456
    assert ucd.ucd_workspace_size(L, ucd.FWD, ucd.ALGO_IM2COL, 9) == ucd.WS_NA      # b > N
    # Winograd: 64 bytes x (C*K + b*T*(C+K)), T = 8*8 tiles: 32 + 64 + 128 KiB at b = 1
    assert ucd.ucd_workspace_size(L, ucd.FWD, ucd.ALGO_WINOGRAD, 1) == 64 * (16 * 32 + 64 * 48) == 224 * 1024
    assert ucd.ucd_workspace_size(L, ucd.BWD_DATA, ucd.ALGO_WINOGRAD, 2) == 64 * (16 * 32 + 128 * 48)
    assert ucd.ucd_workspace_size(L, ucd.BWD_FILTER, ucd.ALGO_WINOGRAD, 1) == 64 * (16 * 32 + 64 * 48)
    # Winograd F(4x4,3x3): 36 planes of 4 bytes, T = 4*4 tiles
    assert ucd.ucd_workspace_size(L, ucd.FWD, ucd.ALGO_WINOGRAD4, 1) == 144 * (16 * 32 + 16 * 48)
    assert ucd.ucd_workspace_size(L, ucd.BWD_DATA, ucd.ALGO_WINOGRAD4, 3) == 144 * (16 * 32 + 48 * 48)
    assert ucd.ucd_workspace_size(L, ucd.BWD_FILTER, ucd.ALGO_WINOGRAD4, 2) == 144 * (16 * 32 + 32 * 48)
    # FFT: 144 planes of 4 bytes, 14 x 14 output tiles: T = 2*2, 2C*2K + ld*(2C + 2K)
    assert ucd.ucd_workspace_size(L, ucd.FWD, ucd.ALGO_FFT, 3) == 4 * 144 * (32 * 64 + 12 * 96)
    assert ucd.ucd_workspace_size(L, ucd.BWD_FILTER, ucd.ALGO_FFT, 1) == 4 * 144 * (4 * 32 * 16 + 4 * 96)
    # fused Winograd: the transformed filter, 64 bytes x Ci (rounded up to 8) x Co (rounded up to 4)
    assert ucd.ucd_workspace_size(L, ucd.FWD, ucd.ALGO_WINOGRAD_FUSED, 8) == 64 * 16 * 32
    assert ucd.ucd_workspace_size(L, ucd.BWD_FILTER, ucd.ALGO_WINOGRAD_FUSED, 8) == 64 * 16 * 32
    Lc3 = ucd.layer(N=8, C=3, H=16, W=16, K=30, R=3, S=3, pad_h=1, pad_w=1)
    assert ucd.ucd_workspace_size(Lc3, ucd.FWD, ucd.ALGO_WINOGRAD_FUSED, 1) == 64 * 8 * 32
    assert ucd.ucd_workspace_size(Lc3, ucd.BWD_DATA, ucd.ALGO_WINOGRAD_FUSED, 1) == 64 * 32 * 4
    # strided BackwardData with three taps per phase and axis: a 3x3 convolution from K to C * stride^2 channels
    L11s4 = ucd.layer(N=4, C=3, H=35, W=35, K=20, R=11, S=11, pad_h=2, pad_w=2, stride_h=4, stride_w=4)
    assert ucd.ucd_workspace_size(L11s4, ucd.BWD_DATA, ucd.ALGO_WINOGRAD_FUSED, 4) == 64 * 24 * 48
    assert ucd.ucd_workspace_size(L11s4, ucd.FWD, ucd.ALGO_WINOGRAD_FUSED, 4) == ucd.WS_NA
    assert ucd.ucd_workspace_size(L11s4, ucd.BWD_FILTER, ucd.ALGO_WINOGRAD_FUSED, 4) == ucd.WS_NA
    # mirrored filter copy: BackwardData of stride-1 layers only, the filter's own size (16-byte multiple)
    assert ucd.ucd_workspace_size(L, ucd.BWD_DATA, ucd.ALGO_IMPLICIT_MIRROR, 5) == 4 * 32 * 16 * 9
    assert ucd.ucd_workspace_size(L, ucd.FWD, ucd.ALGO_IMPLICIT_MIRROR, 5) == ucd.WS_NA
    assert ucd.ucd_workspace_size(L, ucd.BWD_FILTER, ucd.ALGO_IMPLICIT_MIRROR, 5) == ucd.WS_NA
    Lb = ucd.layer(N=8, C=3, H=16, W=16, K=5, R=3, S=3, pad_h=1, pad_w=1, dtype=1)
    assert ucd.ucd_workspace_size(Lb, ucd.BWD_DATA, ucd.ALGO_IMPLICIT_MIRROR, 1) == 272   # 2 x 135 -> 16-byte multiple
    # Winograd F(2x2,5x5), fused: 36 planes of the transformed filter (Ci rounded up to 8, Co to 4);
    # BackwardFilter: the 36 K x C product planes; 5x5 stride-1 layers with horizontal padding 2, fp32
    L5 = ucd.layer(N=8, C=20, H=16, W=16, K=30, R=5, S=5, pad_h=2, pad_w=2)
    assert ucd.ucd_workspace_size(L5, ucd.FWD, ucd.ALGO_WINOGRAD5_FUSED, 8) == 144 * 24 * 32
    assert ucd.ucd_workspace_size(L5, ucd.BWD_DATA, ucd.ALGO_WINOGRAD5_FUSED, 3) == 144 * 32 * 20
    assert ucd.ucd_workspace_size(L5, ucd.BWD_FILTER, ucd.ALGO_WINOGRAD5_FUSED, 1) == 144 * 30 * 20
    assert ucd.ucd_workspace_size(L, ucd.FWD, ucd.ALGO_WINOGRAD5_FUSED, 1) == ucd.WS_NA          # 3x3
    assert ucd.ucd_workspace_size(ucd.layer(N=8, C=20, H=16, W=16, K=30, R=5, S=5, pad_h=2, pad_w=1),
                                  ucd.FWD, ucd.ALGO_WINOGRAD5_FUSED, 1) == ucd.WS_NA             # padding 1
    assert ucd.ucd_workspace_size(ucd.layer(N=8, C=20, H=16, W=16, K=30, R=5, S=5, pad_h=2, pad_w=2, dtype=1),
                                  ucd.FWD, ucd.ALGO_WINOGRAD5_FUSED, 1) == ucd.WS_NA             # bf16
    Ls2 = ucd.layer(N=8, C=16, H=16, W=16, K=32, R=3, S=3, pad_h=1, pad_w=1, stride_h=2, stride_w=2)
    assert ucd.ucd_workspace_size(Ls2, ucd.BWD_FILTER, ucd.ALGO_WINOGRAD, 1) == ucd.WS_NA  # stride 2
    assert ucd.ucd_workspace_size(Ls2, ucd.BWD_DATA, ucd.ALGO_IMPLICIT_MIRROR, 1) == ucd.WS_NA
    assert ucd.ucd_workspace_size(Ls2, ucd.BWD_DATA, ucd.ALGO_WINOGRAD_FUSED, 1) == ucd.WS_NA  # two taps per phase
    L11 = ucd.layer(N=4, C=8, H=7, W=7, K=8, R=1, S=1)
    assert ucd.ucd_workspace_size(L11, ucd.FWD, ucd.ALGO_IM2COL, 1) == ucd.WS_NA    # col == x
    assert ucd.ucd_workspace_size(L11, ucd.FWD, ucd.ALGO_WINOGRAD, 1) == ucd.WS_NA  # not 3x3
    bad = ucd.layer(N=4, C=8, H=2, W=2, K=8, R=5, S=5)
    assert ucd.ucd_workspace_size(bad, ucd.FWD, ucd.ALGO_IMPLICIT, 1) == ucd.WS_NA


def test_plan_fixed_validation_and_query():
    import pytest
    L = ucd.layer(N=8, C=16, H=16, W=16, K=32, R=3, S=3, pad_h=1, pad_w=1)
    p = ucd.ucd_plan_fixed(L, ucd.FWD, [(0, 3), (1, 5)])
    assert p.query() == ([(0, 3), (1, 5)], 0, 5 * 147456)
    for micro, status in (([(0, 3), (0, 4)], ucd.E_INVALID), ([(0, 0), (0, 8)], ucd.E_INVALID),
                          ([(ucd.N_ALGO, 8)], ucd.E_INVALID)):
        with pytest.raises(ucd.UcdError) as e:
            ucd.ucd_plan_fixed(L, ucd.FWD, micro)
        assert e.value.status == status


def test_execution_rejects_bad_calls_before_any_launch():
    import pytest
    L = ucd.layer(N=8, C=16, H=16, W=16, K=32, R=3, S=3, pad_h=1, pad_w=1)
    p = ucd.ucd_plan_fixed(L, ucd.FWD, [(1, 8)])
    lib = ucd.lib()
    # null tensors
    assert lib.ucd_conv_fwd(p.handle, None, None, None, None, 0, None) == ucd.E_NULLPTR
    # workspace one byte short (fake non-null addresses are never dereferenced on this path)
    assert lib.ucd_conv_fwd(p.handle, 4096, 4096, 4096, 4096, 8 * 147456 - 1, None) == ucd.E_WS_TOO_SMALL
    # wrong operation for this plan
    assert lib.ucd_conv_bwd_data(p.handle, 4096, 4096, 4096, 4096, 1 << 30, None) == ucd.E_INVALID
    pf = ucd.ucd_plan_fixed(L, ucd.BWD_FILTER, [(0, 8)])
    assert lib.ucd_conv_bwd_filter(pf.handle, 4096, 4096, 4096, 0.5, None, 0, None) == ucd.E_INVALID
    # a table plan has no layer attached
    t = [[ucd.TIME_INF, 5, 9]]
    pt = ucd.ucd_plan_from_table(2, 0, ucd.POLICY_ALL, t, [[ucd.WS_NA, 0, 0]])
    assert lib.ucd_conv_fwd(pt.handle, 4096, 4096, 4096, None, 0, None) == ucd.E_INVALID


def test_run_micro_rejects_a_micro_batch_beyond_the_descriptor():
    """The descriptor's N is the extent of the caller's buffers: b > N (or b < 1) is an error
    before anything is launched, and so is a bf16 tensor pointer that is not 2-byte aligned."""
    import ctypes as C
    L = ucd.layer(N=8, C=16, H=16, W=16, K=32, R=3, S=3, pad_h=1, pad_w=1)
    lib = ucd.lib()
    for b in (0, 9, 1 << 20):
        assert lib.ucd_run_micro(C.byref(L), ucd.FWD, ucd.ALGO_IMPLICIT, b, 4096, 4096, 4096, 0.0,
                                 None, 0, None) == ucd.E_INVALID
    Lh = ucd.layer(N=8, C=16, H=16, W=16, K=32, R=3, S=3, pad_h=1, pad_w=1, dtype=1)
    assert lib.ucd_run_micro(C.byref(Lh), ucd.FWD, ucd.ALGO_IMPLICIT, 8, 4097, 4096, 4096, 0.0,
                             None, 0, None) == ucd.E_INVALID
    Lbad = ucd.layer(N=8, C=16, H=16, W=16, K=32, R=3, S=3, pad_h=1, pad_w=1, dtype=2)
    assert lib.ucd_run_micro(C.byref(Lbad), ucd.FWD, ucd.ALGO_IMPLICIT, 8, 4096, 4096, 4096, 0.0,
                             None, 0, None) == ucd.E_INVALID


def test_reproducible_mode_workspace_sizes():
    """In the reproducible mode BackwardFilter is the implicit GEMM's alone and needs one K*C*R*S
    plane per reduction chunk; Forward / BackwardData sizes do not change."""
    L = ucd.layer(N=64, C=64, H=28, W=28, K=96, R=3, S=3, pad_h=1, pad_w=1)
    before = [[ucd.ucd_workspace_size(L, op, a, 64) for a in range(ucd.N_ALGO)] for op in range(3)]
    assert before[ucd.BWD_FILTER][ucd.ALGO_IMPLICIT] == 0
    assert ucd.ucd_set_deterministic(1) == 0
    try:
        assert ucd.ucd_set_deterministic(-1) == 1
        after = [[ucd.ucd_workspace_size(L, op, a, 64) for a in range(ucd.N_ALGO)] for op in range(3)]
        assert after[ucd.FWD] == before[ucd.FWD] and after[ucd.BWD_DATA] == before[ucd.BWD_DATA]
        need = after[ucd.BWD_FILTER][ucd.ALGO_IMPLICIT]
        plane = 4 * 96 * 64 * 9
        assert need % plane == 0 and 2 <= need // plane and need <= 32 << 20
        assert all(after[ucd.BWD_FILTER][a] == ucd.WS_NA for a in range(1, ucd.N_ALGO))
    finally:
        assert ucd.ucd_set_deterministic(0) == 1
    assert [[ucd.ucd_workspace_size(L, op, a, 64) for a in range(ucd.N_ALGO)] for op in range(3)] == before
