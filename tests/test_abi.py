"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, sizes follow the packed format, and bad arguments are refused
on the host before anything is launched (no GPU needed)."""

import ctypes
import os
import re

import pytest

from paper_1605_04711_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "twn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(twn_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = api.lib()
    names = header_functions()
    assert len(names) >= 13
    for n in names:
        assert hasattr(L, n), n
    assert sorted(api.EXPORTS) == names
    assert L.twn_abi_version() == 2
    assert api.status_str(0) == "ok" and api.status_str(-3).startswith("misaligned")


def test_packed_sizes():
    assert api.twn_packed_words_per_row(1) == 8
    assert api.twn_packed_words_per_row(128) == 8
    assert api.twn_packed_words_per_row(129) == 16
    assert api.twn_packed_words_per_row(0) == 0
    assert api.twn_packed_bytes(64, 1152) * 16 == 64 * 1152 * 4      # 2 bits per weight
    assert api.twn_packed_bytes(10, 27) == 10 * 32


FAKE = ctypes.c_void_p(0x10000)       # aligned, never dereferenced: every call below fails validation first
ODD = ctypes.c_void_p(0x10004)


def test_ternarize_argument_errors():
    L = api.lib()
    wd = api.WeightDesc(8, 16, 3, 3)
    ws = L.twn_ternarize_workspace_bytes(ctypes.byref(wd), 1)
    assert ws > 0
    call = lambda *a: L.twn_ternarize(*a)
    ok_args = [FAKE, ctypes.byref(wd), 1, ctypes.c_float(0.7), FAKE, None, FAKE, FAKE, FAKE, FAKE, ws, None]
    a = list(ok_args); a[0] = None
    assert call(*a) == -1
    a = list(ok_args); a[4] = None
    assert call(*a) == -1
    a = list(ok_args); a[2] = 3                      # groups must divide rows
    assert call(*a) == -2
    a = list(ok_args); a[3] = ctypes.c_float(0.0)    # factor in (0, 1]
    assert call(*a) == -2
    a = list(ok_args); a[1] = ctypes.byref(api.WeightDesc(0, 16, 3, 3))
    assert call(*a) == -2
    a = list(ok_args); a[0] = ODD
    assert call(*a) == -3
    a = list(ok_args); a[10] = ws - 1
    assert call(*a) == -5
    a = list(ok_args); a[9] = None
    assert call(*a) == -5


def test_ternarize_static_argument_errors():
    # every check that needs no GPU comes before the first GPU call of the entry point
    L = api.lib()
    wd = api.WeightDesc(8, 16, 3, 3)
    assert L.twn_ternarize_static_scratch_bytes() == 98304
    ok_args = [FAKE, ctypes.byref(wd), 1, ctypes.c_float(0.7), FAKE, None, FAKE, FAKE, FAKE, None]
    call = lambda *a: L.twn_ternarize_static(*a)
    a = list(ok_args); a[0] = None
    assert call(*a) == -1
    a = list(ok_args); a[2] = 3
    assert call(*a) == -2
    a = list(ok_args); a[4] = ODD
    assert call(*a) == -3
    big = api.WeightDesc(1 << 20, 1 << 20, 1, 1)     # 2^40 weights: beyond what the fixed array is specified for
    a = list(ok_args); a[1] = ctypes.byref(big)
    assert call(*a) == -2


def test_gemm_and_conv_argument_errors():
    L = api.lib()
    d = api.GemmDesc(64, 32, 128, api.TWN_BF16, api.TWN_BF16, api.TWN_VAR_BF16_POSTSCALE, 0, 0, 1)
    assert L.twn_gemm_fwd(ctypes.byref(d), None, FAKE, FAKE, None, FAKE, None, 0, None) == -1
    bad = api.GemmDesc(0, 32, 128, 1, 1, 0, 0, 0, 1)
    assert L.twn_gemm_fwd(ctypes.byref(bad), FAKE, FAKE, FAKE, None, FAKE, None, 0, None) == -2
    bad = api.GemmDesc(64, 32, 128, 1, 1, 0, 64, 0, 1)       # ldx < K
    assert L.twn_gemm_fwd(ctypes.byref(bad), FAKE, FAKE, FAKE, None, FAKE, None, 0, None) == -2
    bad = api.GemmDesc(64, 32, 128, api.TWN_F32, 1, api.TWN_VAR_BF16_POSTSCALE, 0, 0, 1)   # variant/dtype mismatch
    assert L.twn_gemm_fwd(ctypes.byref(bad), FAKE, FAKE, FAKE, None, FAKE, None, 0, None) == -4
    bad = api.GemmDesc(64, 32, 128, 1, 1, 0, 0, 0, 5)        # alpha groups must divide N
    assert L.twn_gemm_fwd(ctypes.byref(bad), FAKE, FAKE, FAKE, None, FAKE, None, 0, None) == -2
    assert L.twn_gemm_fwd(ctypes.byref(d), ODD, FAKE, FAKE, None, FAKE, None, 0, None) == -3

    c = api.ConvDesc(2, 8, 8, 16, 32, 3, 3, 1, 1, 1, 1, 1, 1, 1, 1, 0, 1)
    assert L.twn_conv2d_fwd(ctypes.byref(c), FAKE, None, FAKE, None, FAKE, None, 0, None) == -1
    bad = api.ConvDesc(2, 2, 2, 16, 32, 5, 5, 1, 1, 0, 0, 1, 1, 1, 1, 0, 1)    # empty output
    assert L.twn_conv2d_fwd(ctypes.byref(bad), FAKE, FAKE, FAKE, None, FAKE, None, 0, None) == -2
    bad = api.ConvDesc(2, 8, 8, 16, 32, 3, 3, 0, 1, 1, 1, 1, 1, 1, 1, 0, 1)    # stride 0
    assert L.twn_conv2d_fwd(ctypes.byref(bad), FAKE, FAKE, FAKE, None, FAKE, None, 0, None) == -2
    assert L.twn_conv2d_fwd(ctypes.byref(c), FAKE, ODD, FAKE, None, FAKE, None, 0, None) == -3

    # two convolutions over one input: both descriptors are checked before any launch
    c3 = api.ConvDesc(2, 8, 8, 16, 32, 3, 3, 2, 2, 1, 1, 1, 1, 1, 1, 0, 1)
    c1 = api.ConvDesc(2, 8, 8, 16, 32, 1, 1, 2, 2, 0, 0, 1, 1, 1, 1, 0, 1)
    pair = lambda a, b, x=FAKE, w0=FAKE, y1=FAKE: L.twn_conv2d_fwd_pair(
        ctypes.byref(a), ctypes.byref(b), x, w0, FAKE, None, FAKE, FAKE, FAKE, None, y1, None)
    assert pair(c3, c1, x=None) == -1
    assert pair(c3, c1, y1=None) == -1
    other = api.ConvDesc(2, 8, 8, 32, 32, 1, 1, 2, 2, 0, 0, 1, 1, 1, 1, 0, 1)            # another channel count
    assert pair(c3, other) == -2
    c12 = api.ConvDesc(2, 8, 8, 12, 32, 1, 1, 2, 2, 0, 0, 1, 1, 1, 1, 0, 1)             # C % 8 != 0
    assert pair(c12, c12) == -4
    f32 = api.ConvDesc(2, 8, 8, 16, 32, 1, 1, 2, 2, 0, 0, 1, 1, api.TWN_F32, api.TWN_F32, api.TWN_VAR_FP32, 1)
    assert pair(c3, f32) == -4
    assert pair(c3, c1, w0=ODD) == -3

    ws = L.twn_conv2d_bwd_ste_workspace_bytes(ctypes.byref(c))
    assert ws > 0
    f0 = ctypes.c_float(0.0)
    assert L.twn_conv2d_bwd_ste(ctypes.byref(c), FAKE, None, FAKE, FAKE, FAKE, FAKE, None, f0, FAKE, ws, None) == -1
    assert L.twn_conv2d_bwd_ste(ctypes.byref(c), FAKE, FAKE, None, FAKE, FAKE, FAKE, None, f0, FAKE, ws, None) == -1
    assert L.twn_conv2d_bwd_ste(ctypes.byref(c), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, f0, FAKE, ws - 1, None) == -5
    assert L.twn_conv2d_bwd_ste(ctypes.byref(c), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, ctypes.c_float(0.5),
                                FAKE, ws, None) == -4


def test_missing_library_is_loud(monkeypatch):
    monkeypatch.setattr(api, "_lib", None)
    monkeypatch.setattr(api, "_LIB_PATH", "/nonexistent/libtwn.so")
    with pytest.raises(FileNotFoundError):
        api.lib()


def test_output_and_residual_alignment_is_validated():
    # rows with channel counts in multiples of 8 are written with 16-byte stores: Y and the residual must be 16-byte aligned
    L = api.lib()
    d = api.GemmDesc(64, 32, 128, api.TWN_BF16, api.TWN_BF16, api.TWN_VAR_BF16_POSTSCALE, 0, 0, 1)
    Y2 = ctypes.c_void_p(0x10002)
    assert L.twn_gemm_fwd(ctypes.byref(d), FAKE, FAKE, FAKE, None, Y2, None, 0, None) == -3
    ep = api.Epilogue(None, None, 0x10008, 0)
    assert L.twn_gemm_fwd(ctypes.byref(d), FAKE, FAKE, FAKE, ctypes.byref(ep), FAKE, None, 0, None) == -3
    c = api.ConvDesc(1, 8, 8, 16, 32, 3, 3, 1, 1, 1, 1, 1, 1, api.TWN_BF16, api.TWN_BF16, api.TWN_VAR_BF16_POSTSCALE, 1)
    assert L.twn_conv2d_fwd(ctypes.byref(c), FAKE, FAKE, FAKE, None, Y2, None, 0, None) == -3
    assert L.twn_conv2d_bwd_ste(ctypes.byref(c), None, FAKE, FAKE, FAKE, Y2, None, None, ctypes.c_float(0.0),
                                None, 0, None) == -3
    # odd channel counts are stored element by element: 2-byte alignment is enough (the call then fails later,
    # on the missing workspace or not at all; it must not fail on alignment)
    c2 = api.ConvDesc(1, 8, 8, 16, 30, 3, 3, 1, 1, 1, 1, 1, 1, api.TWN_BF16, api.TWN_BF16, api.TWN_VAR_BF16_POSTSCALE, 1)
    assert L.twn_conv2d_bwd_ste(ctypes.byref(c2), None, FAKE, FAKE, FAKE, None, None, None, ctypes.c_float(0.0),
                                None, 0, None) != -3
