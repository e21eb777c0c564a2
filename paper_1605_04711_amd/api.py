"""ctypes binding of libtwn.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/twn.h).
PyTorch supplies device memory (`torch.empty(..., device='cuda')`), pointers
(`.data_ptr()`) and the current HIP stream; all arithmetic runs in the library's
kernels.  There is no fallback: a missing library raises.
"""

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

TWN_F32, TWN_BF16 = 0, 1
TWN_VAR_BF16_POSTSCALE, TWN_VAR_BF16_ALPHA_LDS, TWN_VAR_I8_STORED_POSTSCALE, TWN_VAR_FP32 = 0, 1, 2, 3
TWN_VAR_BF16_SIGN1_POSTSCALE = 4
TWN_VAR_ADDSUB_SPARSE = 5

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtwn.so")
_lib = None

EXPORTS = [
    "twn_status_str", "twn_reload_env", "twn_abi_version", "twn_packed_words_per_row", "twn_packed_bytes",
    "twn_ternarize_workspace_bytes", "twn_ternarize", "twn_ternarize_static_scratch_bytes", "twn_ternarize_static",
    "twn_ternarize_batch_workspace_bytes", "twn_ternarize_batch",
    "twn_unpack_i8",
    "twn_gemm_fwd_workspace_bytes", "twn_gemm_fwd",
    "twn_conv2d_fwd_workspace_bytes", "twn_conv2d_fwd", "twn_conv2d_fwd_pair",
    "twn_conv2d_bwd_ste_workspace_bytes", "twn_conv2d_bwd_ste",
    "twn_sgd_update", "twn_ternarize_presummed",
    "twn_packed1_words_per_row", "twn_binarize_workspace_bytes", "twn_binarize",
]


class TwnError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, status_str(status), status))


class WeightDesc(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int32), ("C", ctypes.c_int32), ("R", ctypes.c_int32), ("S", ctypes.c_int32)]


class TernarizeItem(ctypes.Structure):
    _fields_ = [("W", ctypes.c_void_p), ("wd", WeightDesc), ("packed", ctypes.c_void_p), ("packed_T", ctypes.c_void_p),
                ("delta", ctypes.c_void_p), ("alpha", ctypes.c_void_p), ("nnz", ctypes.c_void_p),
                ("groups", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class GemmDesc(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int32), ("K", ctypes.c_int32),
                ("x_dtype", ctypes.c_int32), ("y_dtype", ctypes.c_int32), ("variant", ctypes.c_int32),
                ("ldx", ctypes.c_int64), ("ldy", ctypes.c_int64), ("alpha_groups", ctypes.c_int32)]


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "H", "W", "C", "O", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w",
                 "x_dtype", "y_dtype", "variant", "alpha_groups")]


class Epilogue(ctypes.Structure):
    _fields_ = [("scale", ctypes.c_void_p), ("shift", ctypes.c_void_p), ("residual", ctypes.c_void_p),
                ("relu", ctypes.c_int32)]


def library_path():
    return _LIB_PATH


def lib():
    """Load libtwn.so (built by `python -m paper_1605_04711_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_1605_04711_amd.build`" % _LIB_PATH)
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, sz, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_float
        L.twn_status_str.restype = ctypes.c_char_p
        L.twn_status_str.argtypes = [i32]
        L.twn_abi_version.restype = i32
        L.twn_packed_words_per_row.restype = i64
        L.twn_packed_words_per_row.argtypes = [i64]
        L.twn_packed_bytes.restype = sz
        L.twn_packed_bytes.argtypes = [i32, i64]
        L.twn_ternarize_workspace_bytes.restype = sz
        L.twn_ternarize_workspace_bytes.argtypes = [ctypes.POINTER(WeightDesc), i32]
        L.twn_ternarize.restype = i32
        L.twn_ternarize.argtypes = [vp, ctypes.POINTER(WeightDesc), i32, f32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.twn_ternarize_static_scratch_bytes.restype = sz
        L.twn_ternarize_static_scratch_bytes.argtypes = []
        L.twn_ternarize_static.restype = i32
        L.twn_ternarize_static.argtypes = [vp, ctypes.POINTER(WeightDesc), i32, f32, vp, vp, vp, vp, vp, vp]
        L.twn_ternarize_batch_workspace_bytes.restype = sz
        L.twn_ternarize_batch_workspace_bytes.argtypes = [i32]
        L.twn_ternarize_batch.restype = i32
        L.twn_ternarize_batch.argtypes = [ctypes.POINTER(TernarizeItem), i32, f32, vp, sz, vp]
        L.twn_unpack_i8.restype = i32
        L.twn_unpack_i8.argtypes = [vp, i32, i64, vp, vp]
        L.twn_reload_env.restype = None
        L.twn_reload_env.argtypes = []
        L.twn_packed1_words_per_row.restype = i64
        L.twn_packed1_words_per_row.argtypes = [i64]
        L.twn_binarize_workspace_bytes.restype = sz
        L.twn_binarize_workspace_bytes.argtypes = [ctypes.POINTER(WeightDesc), i32]
        L.twn_binarize.restype = i32
        L.twn_binarize.argtypes = [vp, ctypes.POINTER(WeightDesc), i32, vp, vp, vp, sz, vp]
        L.twn_sgd_update.restype = i32
        L.twn_sgd_update.argtypes = [vp, vp, vp, i64, f32, f32, f32, vp, sz, vp]
        L.twn_ternarize_presummed.restype = i32
        L.twn_ternarize_presummed.argtypes = [vp, ctypes.POINTER(WeightDesc), f32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.twn_gemm_fwd_workspace_bytes.restype = sz
        L.twn_gemm_fwd_workspace_bytes.argtypes = [ctypes.POINTER(GemmDesc)]
        L.twn_gemm_fwd.restype = i32
        L.twn_gemm_fwd.argtypes = [ctypes.POINTER(GemmDesc), vp, vp, vp, ctypes.POINTER(Epilogue), vp, vp, sz, vp]
        L.twn_conv2d_fwd_workspace_bytes.restype = sz
        L.twn_conv2d_fwd_workspace_bytes.argtypes = [ctypes.POINTER(ConvDesc)]
        L.twn_conv2d_fwd.restype = i32
        L.twn_conv2d_fwd.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp, ctypes.POINTER(Epilogue), vp, vp, sz, vp]
        L.twn_conv2d_fwd_pair.restype = i32
        L.twn_conv2d_fwd_pair.argtypes = [ctypes.POINTER(ConvDesc), ctypes.POINTER(ConvDesc), vp,
                                          vp, vp, ctypes.POINTER(Epilogue), vp, vp, vp, ctypes.POINTER(Epilogue), vp, vp]
        L.twn_conv2d_bwd_ste_workspace_bytes.restype = sz
        L.twn_conv2d_bwd_ste_workspace_bytes.argtypes = [ctypes.POINTER(ConvDesc)]
        L.twn_conv2d_bwd_ste.restype = i32
        L.twn_conv2d_bwd_ste.argtypes = [ctypes.POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, vp, f32, vp, sz, vp]
        _lib = L
    return _lib


def status_str(status):
    return lib().twn_status_str(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise TwnError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return TWN_F32
    if t.dtype == torch.bfloat16:
        return TWN_BF16
    raise TypeError("only float32 and bfloat16 tensors are accepted")


def _workspace(nbytes, device, stream=None):
    """Scratch tensor for one call.  Allocated under the stream the kernels are enqueued on, so that the
    caching allocator cannot hand the block to later work of another stream while they still use it."""
    if stream is None:
        return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)
    with torch.cuda.stream(stream):
        return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def _need_contiguous(**tensors):
    for name, t in tensors.items():
        if t is not None and not t.is_contiguous():
            raise TypeError("%s must be contiguous (activations are read as dense NHWC)" % name)


def twn_packed_words_per_row(k):
    return int(lib().twn_packed_words_per_row(int(k)))


def twn_packed_bytes(rows, k):
    return int(lib().twn_packed_bytes(int(rows), int(k)))


@dataclass
class TernaryWeights:
    """Device-resident result of twn_ternarize for one filter bank [rows][C][R][S]."""
    rows: int
    C: int
    R: int
    S: int
    groups: int
    packed: torch.Tensor                 # uint32 viewed as int32 [rows][words_per_row(R*S*C)]
    packed_T: Optional[torch.Tensor]     # [C][words_per_row(R*S*rows)] or None
    delta: torch.Tensor                  # float32 [groups]
    alpha: torch.Tensor                  # float32 [groups]
    nnz: torch.Tensor                    # int64 [groups]
    codes_i8: Optional[torch.Tensor] = None   # int8 [rows][K], the weights of TWN_VAR_I8_STORED_POSTSCALE

    @property
    def K(self):
        return self.R * self.S * self.C

    def weights_for(self, variant):
        """Device tensor a forward call reads as its `weights` argument."""
        if variant == TWN_VAR_BF16_SIGN1_POSTSCALE:
            raise ValueError("TWN_VAR_BF16_SIGN1_POSTSCALE reads the 1-bit codes of twn_binarize")
        if variant != TWN_VAR_I8_STORED_POSTSCALE:
            return self.packed
        if self.codes_i8 is None:
            self.codes_i8 = twn_unpack_i8(self.packed, self.rows, self.K)
        return self.codes_i8


def twn_ternarize(W, delta_factor=0.7, groups=1, transposed=False, out=None, workspace=None, stream=None):
    """W: float32 CUDA tensor [rows][C][R][S] (or [rows][K] for a fully-connected layer)."""
    if W.dim() == 2:
        rows, c = W.shape
        r = s = 1
    else:
        rows, c, r, s = W.shape
    if not W.is_contiguous() or W.dtype != torch.float32 or not W.is_cuda:
        raise TypeError("W must be a contiguous float32 CUDA tensor")
    L = lib()
    wd = WeightDesc(rows, c, r, s)
    dev = W.device
    if out is None:
        k, kt = r * s * c, r * s * rows
        packed = torch.empty((rows, twn_packed_words_per_row(k)), dtype=torch.int32, device=dev)
        packed_t = torch.empty((c, twn_packed_words_per_row(kt)), dtype=torch.int32, device=dev) if transposed else None
        out = TernaryWeights(rows, c, r, s, groups, packed, packed_t,
                             torch.empty(groups, dtype=torch.float32, device=dev),
                             torch.empty(groups, dtype=torch.float32, device=dev),
                             torch.empty(groups, dtype=torch.int64, device=dev))
    if workspace is None:
        workspace = _workspace(L.twn_ternarize_workspace_bytes(ctypes.byref(wd), groups), dev, stream)
    rc = L.twn_ternarize(_ptr(W), ctypes.byref(wd), groups, ctypes.c_float(delta_factor),
                         _ptr(out.packed), _ptr(out.packed_T), _ptr(out.delta), _ptr(out.alpha), _ptr(out.nnz),
                         _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "twn_ternarize")
    return out


def reload_env():
    """Have the library read its TWN_* tuning overrides again (they are read once and remembered)."""
    lib().twn_reload_env()


@dataclass
class BinaryWeights:
    """Device-resident result of twn_binarize: 1-bit sign codes and the scale(s) of the binary-weight comparison.
    Passed to the forward calls with variant=TWN_VAR_BF16_SIGN1_POSTSCALE."""
    rows: int
    C: int
    R: int
    S: int
    groups: int
    packed: torch.Tensor                 # uint32 viewed as int32 [rows][packed1_words_per_row(R*S*C)]
    alpha: torch.Tensor                  # float32 [groups]

    @property
    def K(self):
        return self.R * self.S * self.C

    def weights_for(self, variant):
        if variant != TWN_VAR_BF16_SIGN1_POSTSCALE:
            raise ValueError("sign codes are read by TWN_VAR_BF16_SIGN1_POSTSCALE only")
        return self.packed


def twn_binarize(W, groups=1, workspace=None, stream=None):
    """Sign codes and alpha = mean|W| per group of a float32 CUDA tensor [rows][C][R][S] (or [rows][K])."""
    if W.dim() == 2:
        rows, c = W.shape
        r = s = 1
    else:
        rows, c, r, s = W.shape
    if not W.is_contiguous() or W.dtype != torch.float32 or not W.is_cuda:
        raise TypeError("W must be a contiguous float32 CUDA tensor")
    L = lib()
    wd = WeightDesc(rows, c, r, s)
    out = BinaryWeights(rows, c, r, s, groups,
                        torch.empty((rows, int(L.twn_packed1_words_per_row(r * s * c))), dtype=torch.int32, device=W.device),
                        torch.empty(groups, dtype=torch.float32, device=W.device))
    if workspace is None:
        workspace = _workspace(L.twn_binarize_workspace_bytes(ctypes.byref(wd), groups), W.device, stream)
    rc = L.twn_binarize(_ptr(W), ctypes.byref(wd), groups, _ptr(out.packed), _ptr(out.alpha), _ptr(workspace),
                        workspace.numel(), _stream(stream))
    _check(rc, "twn_binarize")
    return out


def twn_sgd_update(W, V, dW, lr, momentum=0.9, weight_decay=1e-4, tern_workspace=None, stream=None):
    """In-place SGD step on the float32 weights W with velocity V and gradient dW (all contiguous float32 CUDA
    tensors of one shape).  With `tern_workspace` (a uint8 tensor of twn_ternarize's workspace size) the pass-1 sums
    of the next ternarization are left there for twn_ternarize(..., presummed=True)."""
    for name, t in (("W", W), ("V", V), ("dW", dW)):
        if not t.is_contiguous() or t.dtype != torch.float32 or not t.is_cuda or t.shape != W.shape:
            raise TypeError("%s must be a contiguous float32 CUDA tensor of the shape of W" % name)
    rc = lib().twn_sgd_update(_ptr(W), _ptr(V), _ptr(dW), W.numel(), ctypes.c_float(lr), ctypes.c_float(momentum),
                              ctypes.c_float(weight_decay), _ptr(tern_workspace),
                              tern_workspace.numel() if tern_workspace is not None else 0, _stream(stream))
    _check(rc, "twn_sgd_update")


def twn_ternarize_presummed(W, out, workspace, delta_factor=0.7, stream=None):
    """twn_ternarize (one group) on the weights twn_sgd_update has just updated, using the sums it left in
    `workspace`; `out` is a TernaryWeights with groups == 1."""
    if not W.is_contiguous() or W.dtype != torch.float32 or not W.is_cuda:
        raise TypeError("W must be a contiguous float32 CUDA tensor")
    wd = WeightDesc(out.rows, out.C, out.R, out.S)
    rc = lib().twn_ternarize_presummed(_ptr(W), ctypes.byref(wd), ctypes.c_float(delta_factor),
                                       _ptr(out.packed), _ptr(out.packed_T), _ptr(out.delta), _ptr(out.alpha),
                                       _ptr(out.nnz), _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "twn_ternarize_presummed")
    return out


def twn_ternarize_static(W, out, delta_factor=0.7, stream=None):
    """twn_ternarize without a workspace: every buffer of `out` (a TernaryWeights) is the caller's, and the call
    allocates nothing on the device."""
    if not W.is_contiguous() or W.dtype != torch.float32 or not W.is_cuda:
        raise TypeError("W must be a contiguous float32 CUDA tensor")
    wd = WeightDesc(out.rows, out.C, out.R, out.S)
    rc = lib().twn_ternarize_static(_ptr(W), ctypes.byref(wd), out.groups, ctypes.c_float(delta_factor),
                                    _ptr(out.packed), _ptr(out.packed_T), _ptr(out.delta), _ptr(out.alpha),
                                    _ptr(out.nnz), _stream(stream))
    _check(rc, "twn_ternarize_static")
    return out


def _new_ternary_weights(rows, c, r, s, groups, transposed, dev):
    k, kt = r * s * c, r * s * rows
    packed = torch.empty((rows, twn_packed_words_per_row(k)), dtype=torch.int32, device=dev)
    packed_t = torch.empty((c, twn_packed_words_per_row(kt)), dtype=torch.int32, device=dev) if transposed else None
    return TernaryWeights(rows, c, r, s, groups, packed, packed_t,
                          torch.empty(groups, dtype=torch.float32, device=dev),
                          torch.empty(groups, dtype=torch.float32, device=dev),
                          torch.empty(groups, dtype=torch.int64, device=dev))


def twn_ternarize_batch(Ws, delta_factor=0.7, transposed=False, out=None, workspace=None, stream=None, per_filter=False):
    """Ternarization of up to 32 weight tensors in one call (per layer, or one Delta and alpha per filter with
    per_filter=True; with `out` given, each tensor's own `groups` decides); returns a list of TernaryWeights."""
    L = lib()
    shapes = []
    for W in Ws:
        if not W.is_contiguous() or W.dtype != torch.float32 or not W.is_cuda:
            raise TypeError("every W must be a contiguous float32 CUDA tensor")
        shapes.append(tuple(W.shape) + (1, 1) if W.dim() == 2 else tuple(W.shape))
    dev = Ws[0].device
    if out is None:
        out = [_new_ternary_weights(r_, c, r, s, r_ if per_filter else 1, transposed, dev) for (r_, c, r, s) in shapes]
    items = (TernarizeItem * len(Ws))()
    for i, (W, o, (rows, c, r, s)) in enumerate(zip(Ws, out, shapes)):
        items[i] = TernarizeItem(_ptr(W), WeightDesc(rows, c, r, s), _ptr(o.packed), _ptr(o.packed_T), _ptr(o.delta),
                                 _ptr(o.alpha), _ptr(o.nnz), o.groups, 0)
    if workspace is None:
        workspace = _workspace(L.twn_ternarize_batch_workspace_bytes(len(Ws)), dev, stream)
    rc = L.twn_ternarize_batch(items, len(Ws), ctypes.c_float(delta_factor), _ptr(workspace), workspace.numel(),
                               _stream(stream))
    _check(rc, "twn_ternarize_batch")
    return out


def twn_unpack_i8(packed, rows, k, stream=None):
    codes = torch.empty((rows, k), dtype=torch.int8, device=packed.device)
    _check(lib().twn_unpack_i8(_ptr(packed), rows, k, _ptr(codes), _stream(stream)), "twn_unpack_i8")
    return codes


def _epilogue(scale, shift, residual, relu):
    if scale is None and shift is None and residual is None and not relu:
        return None
    return Epilogue(None if scale is None else scale.data_ptr(), None if shift is None else shift.data_ptr(),
                    None if residual is None else residual.data_ptr(), 1 if relu else 0)


def twn_gemm_fwd_workspace_bytes(m, tw, x_dtype=torch.bfloat16, y_dtype=torch.bfloat16, variant=None):
    if variant is None:
        variant = TWN_VAR_FP32 if x_dtype == torch.float32 else TWN_VAR_BF16_POSTSCALE
    code = {torch.float32: TWN_F32, torch.bfloat16: TWN_BF16}
    d = GemmDesc(m, tw.rows, tw.K, code[x_dtype], code[y_dtype], variant, 0, 0, tw.groups)
    return int(lib().twn_gemm_fwd_workspace_bytes(ctypes.byref(d)))


def twn_gemm_fwd(X, tw, y_dtype=torch.bfloat16, variant=None, scale=None, shift=None, residual=None,
                 relu=False, out=None, workspace=None, stream=None):
    """Y[M][N] = alpha * X[M][K] . W~[N][K]^T; X bf16 (MFMA) or float32 (fp32 variant)."""
    m, k = X.shape
    if k != tw.K:
        raise ValueError("K mismatch")
    if variant is None:
        variant = TWN_VAR_FP32 if X.dtype == torch.float32 else TWN_VAR_BF16_POSTSCALE
    Y = out if out is not None else torch.empty((m, tw.rows), dtype=y_dtype, device=X.device)
    d = GemmDesc(m, tw.rows, k, _dtype_code(X), _dtype_code(Y), variant, X.stride(0), Y.stride(0), tw.groups)
    ep = _epilogue(scale, shift, residual, relu)
    L = lib()
    if workspace is None:
        need = L.twn_gemm_fwd_workspace_bytes(ctypes.byref(d))
        workspace = _workspace(need, X.device, stream) if need else None
    rc = L.twn_gemm_fwd(ctypes.byref(d), _ptr(X), _ptr(tw.weights_for(variant)), _ptr(tw.alpha),
                        None if ep is None else ctypes.byref(ep), _ptr(Y), _ptr(workspace),
                        0 if workspace is None else workspace.numel(), _stream(stream))
    _check(rc, "twn_gemm_fwd")
    return Y


def _conv_desc(x_shape, tw, stride, pad, dil, x_code, y_code, variant):
    n, h, w, c = x_shape
    if c != tw.C:
        raise ValueError("channel mismatch")
    return ConvDesc(n, h, w, c, tw.rows, tw.R, tw.S, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1],
                    x_code, y_code, variant, tw.groups)


def conv_out_shape(x_shape, tw, stride, pad, dil):
    n, h, w, _ = x_shape
    p = (h + 2 * pad[0] - dil[0] * (tw.R - 1) - 1) // stride[0] + 1
    q = (w + 2 * pad[1] - dil[1] * (tw.S - 1) - 1) // stride[1] + 1
    return (n, p, q, tw.rows)


def twn_conv2d_fwd_workspace_bytes(x_shape, tw, stride=(1, 1), pad=(0, 0), dil=(1, 1), x_dtype=torch.bfloat16,
                                   y_dtype=torch.bfloat16, variant=None):
    if variant is None:
        variant = TWN_VAR_FP32 if x_dtype == torch.float32 else TWN_VAR_BF16_POSTSCALE
    code = {torch.float32: TWN_F32, torch.bfloat16: TWN_BF16}
    d = _conv_desc(x_shape, tw, stride, pad, dil, code[x_dtype], code[y_dtype], variant)
    return int(lib().twn_conv2d_fwd_workspace_bytes(ctypes.byref(d)))


def twn_conv2d_fwd(X, tw, stride=(1, 1), pad=(0, 0), dil=(1, 1), y_dtype=torch.bfloat16, variant=None,
                   scale=None, shift=None, residual=None, relu=False, out=None, workspace=None, stream=None):
    """X NHWC; returns Y NHWC [N][P][Q][O]."""
    _need_contiguous(X=X, out=out, residual=residual)
    if variant is None:
        variant = TWN_VAR_FP32 if X.dtype == torch.float32 else TWN_VAR_BF16_POSTSCALE
    Y = out if out is not None else torch.empty(conv_out_shape(X.shape, tw, stride, pad, dil), dtype=y_dtype,
                                                device=X.device)
    d = _conv_desc(X.shape, tw, stride, pad, dil, _dtype_code(X), _dtype_code(Y), variant)
    ep = _epilogue(scale, shift, residual, relu)
    L = lib()
    if workspace is None:
        need = L.twn_conv2d_fwd_workspace_bytes(ctypes.byref(d))
        workspace = _workspace(need, X.device, stream) if need else None
    rc = L.twn_conv2d_fwd(ctypes.byref(d), _ptr(X), _ptr(tw.weights_for(variant)), _ptr(tw.alpha),
                          None if ep is None else ctypes.byref(ep), _ptr(Y), _ptr(workspace),
                          0 if workspace is None else workspace.numel(), _stream(stream))
    _check(rc, "twn_conv2d_fwd")
    return Y


def twn_conv2d_bwd_ste_workspace_bytes(x_shape, tw, stride=(1, 1), pad=(0, 0), dil=(1, 1)):
    d = _conv_desc(x_shape, tw, stride, pad, dil, TWN_BF16, TWN_BF16, TWN_VAR_BF16_POSTSCALE)
    return int(lib().twn_conv2d_bwd_ste_workspace_bytes(ctypes.byref(d)))


def twn_conv2d_bwd_ste(X, dY, tw, stride=(1, 1), pad=(0, 0), dil=(1, 1), need_dx=True, need_dw=True,
                       need_dbias=False, dx_dtype=torch.bfloat16, dW=None, accumulate=False, dX=None,
                       workspace=None, x_shape=None, stream=None, variant=TWN_VAR_BF16_POSTSCALE):
    """Returns (dX or None, dW float32 [O][C][R][S] or None, dbias or None)."""
    xs = tuple(X.shape) if X is not None else tuple(x_shape)
    dev = dY.device
    _need_contiguous(X=X, dY=dY, dX=dX, dW=dW)
    if need_dx and dX is None:
        dX = torch.empty(xs, dtype=dx_dtype, device=dev)
    if need_dw and dW is None:
        dW = torch.empty((tw.rows, tw.C, tw.R, tw.S), dtype=torch.float32, device=dev)
    dbias = torch.empty(tw.rows, dtype=torch.float32, device=dev) if need_dbias else None
    d = _conv_desc(xs, tw, stride, pad, dil, TWN_BF16, _dtype_code(dX) if need_dx else TWN_BF16, variant)
    L = lib()
    if workspace is None:
        workspace = _workspace(L.twn_conv2d_bwd_ste_workspace_bytes(ctypes.byref(d)), dev, stream)
    rc = L.twn_conv2d_bwd_ste(ctypes.byref(d), _ptr(X), _ptr(dY), _ptr(tw.packed_T), _ptr(tw.alpha),
                              _ptr(dX) if need_dx else None, _ptr(dW) if need_dw else None, _ptr(dbias),
                              ctypes.c_float(1.0 if accumulate else 0.0), _ptr(workspace), workspace.numel(),
                              _stream(stream))
    _check(rc, "twn_conv2d_bwd_ste")
    return (dX if need_dx else None), (dW if need_dw else None), dbias


# ---- prepared calls ---------------------------------------------------------------------------------------
# The functions above marshal their arguments on every call (descriptor structs, output shapes, workspace
# queries): several microseconds of host time per call, which shows once a network's layers take ten
# microseconds each.  A prepared call marshals once and returns a function that only makes the C call; the
# tensors it was prepared with are kept alive by the closure.  `stream=None` means torch's current stream at
# call time.

def prepare_conv2d_fwd(X, tw, stride=(1, 1), pad=(0, 0), dil=(1, 1), out=None, variant=None, scale=None, shift=None,
                       residual=None, relu=False, workspace=None):
    if variant is None:
        variant = TWN_VAR_FP32 if X.dtype == torch.float32 else TWN_VAR_BF16_POSTSCALE
    if not X.is_contiguous() or (out is not None and not out.is_contiguous()):
        raise TypeError("X and out must be contiguous NHWC tensors")
    Y = out if out is not None else torch.empty(conv_out_shape(X.shape, tw, stride, pad, dil), dtype=X.dtype,
                                                device=X.device)
    d = _conv_desc(X.shape, tw, stride, pad, dil, _dtype_code(X), _dtype_code(Y), variant)
    ep = _epilogue(scale, shift, residual, relu)
    L = lib()
    if workspace is None:
        need = L.twn_conv2d_fwd_workspace_bytes(ctypes.byref(d))
        workspace = _workspace(need, X.device) if need else None
    fn = L.twn_conv2d_fwd
    args = (ctypes.byref(d), _ptr(X), _ptr(tw.weights_for(variant)), _ptr(tw.alpha),
            None if ep is None else ctypes.byref(ep), _ptr(Y), _ptr(workspace),
            0 if workspace is None else workspace.numel())
    keep = (d, ep, X, Y, tw, scale, shift, residual, workspace)

    def call(stream=None, _keep=keep):
        rc = fn(*args, _stream(stream))
        if rc != 0:
            raise TwnError(rc, "twn_conv2d_fwd")
        return Y
    return call


def prepare_conv2d_fwd_pair(X, tws, geos, outs, scales=(None, None), shifts=(None, None), residuals=(None, None),
                            relus=(False, False)):
    """Two convolutions over the same bf16 NHWC input in one call (a residual block's first convolution and its
    projection shortcut): tws, geos = ((stride, pad, dil), ...), outs and the epilogue tuples have two entries."""
    if not X.is_contiguous() or any(not o.is_contiguous() for o in outs):
        raise TypeError("X and the outputs must be contiguous NHWC tensors")
    ds, eps = [], []
    for tw, (st, pd, dl), Y, sc, sf, rs, rl in zip(tws, geos, outs, scales, shifts, residuals, relus):
        ds.append(_conv_desc(X.shape, tw, st, pd, dl, _dtype_code(X), _dtype_code(Y), TWN_VAR_BF16_POSTSCALE))
        eps.append(_epilogue(sc, sf, rs, rl))
    fn = lib().twn_conv2d_fwd_pair
    args = (ctypes.byref(ds[0]), ctypes.byref(ds[1]), _ptr(X),
            _ptr(tws[0].packed), _ptr(tws[0].alpha), None if eps[0] is None else ctypes.byref(eps[0]), _ptr(outs[0]),
            _ptr(tws[1].packed), _ptr(tws[1].alpha), None if eps[1] is None else ctypes.byref(eps[1]), _ptr(outs[1]))
    keep = (ds, eps, X, tws, outs, scales, shifts, residuals)

    def call(stream=None, _keep=keep):
        rc = fn(*args, _stream(stream))
        if rc != 0:
            raise TwnError(rc, "twn_conv2d_fwd_pair")
        return outs
    return call


def twn_conv2d_fwd_pair(X, tws, geos, scales=(None, None), shifts=(None, None), residuals=(None, None),
                        relus=(False, False), outs=None, stream=None):
    if outs is None:
        outs = tuple(torch.empty(conv_out_shape(X.shape, tw, *g), dtype=torch.bfloat16, device=X.device)
                     for tw, g in zip(tws, geos))
    return prepare_conv2d_fwd_pair(X, tws, geos, outs, scales, shifts, residuals, relus)(stream)


def prepare_gemm_fwd(X, tw, out=None, y_dtype=torch.bfloat16, variant=None, scale=None, shift=None, residual=None,
                     relu=False, workspace=None):
    m, k = X.shape
    if k != tw.K:
        raise ValueError("K mismatch")
    if variant is None:
        variant = TWN_VAR_FP32 if X.dtype == torch.float32 else TWN_VAR_BF16_POSTSCALE
    Y = out if out is not None else torch.empty((m, tw.rows), dtype=y_dtype, device=X.device)
    d = GemmDesc(m, tw.rows, k, _dtype_code(X), _dtype_code(Y), variant, X.stride(0), Y.stride(0), tw.groups)
    ep = _epilogue(scale, shift, residual, relu)
    L = lib()
    if workspace is None:
        need = L.twn_gemm_fwd_workspace_bytes(ctypes.byref(d))
        workspace = _workspace(need, X.device) if need else None
    fn = L.twn_gemm_fwd
    args = (ctypes.byref(d), _ptr(X), _ptr(tw.weights_for(variant)), _ptr(tw.alpha),
            None if ep is None else ctypes.byref(ep), _ptr(Y), _ptr(workspace),
            0 if workspace is None else workspace.numel())
    keep = (d, ep, X, Y, tw, scale, shift, residual, workspace)

    def call(stream=None, _keep=keep):
        rc = fn(*args, _stream(stream))
        if rc != 0:
            raise TwnError(rc, "twn_gemm_fwd")
        return Y
    return call


def prepare_conv2d_bwd_ste(X, dY, tw, stride=(1, 1), pad=(0, 0), dil=(1, 1), dX=None, dW=None, dbias=None,
                           accumulate=False, workspace=None, x_shape=None, variant=TWN_VAR_BF16_POSTSCALE):
    """dX / dW / dbias: the output tensors of the parts wanted (None skips a part)."""
    xs = tuple(X.shape) if X is not None else tuple(x_shape)
    d = _conv_desc(xs, tw, stride, pad, dil, TWN_BF16, _dtype_code(dX) if dX is not None else TWN_BF16, variant)
    L = lib()
    if workspace is None:
        workspace = _workspace(L.twn_conv2d_bwd_ste_workspace_bytes(ctypes.byref(d)), dY.device)
    fn = L.twn_conv2d_bwd_ste
    args = (ctypes.byref(d), _ptr(X), _ptr(dY), _ptr(tw.packed_T), _ptr(tw.alpha), _ptr(dX), _ptr(dW), _ptr(dbias),
            ctypes.c_float(1.0 if accumulate else 0.0), _ptr(workspace), workspace.numel())
    keep = (d, X, dY, tw, dX, dW, dbias, workspace)

    def call(stream=None, _keep=keep):
        rc = fn(*args, _stream(stream))
        if rc != 0:
            raise TwnError(rc, "twn_conv2d_bwd_ste")
    return call


def prepare_ternarize_batch(Ws, out, delta_factor=0.7, workspace=None):
    L = lib()
    items = (TernarizeItem * len(Ws))()
    for i, (W, o) in enumerate(zip(Ws, out)):
        if not W.is_contiguous() or W.dtype != torch.float32 or not W.is_cuda:
            raise TypeError("every W must be a contiguous float32 CUDA tensor")
        items[i] = TernarizeItem(_ptr(W), WeightDesc(o.rows, o.C, o.R, o.S), _ptr(o.packed), _ptr(o.packed_T),
                                 _ptr(o.delta), _ptr(o.alpha), _ptr(o.nnz), o.groups, 0)
    if workspace is None:
        workspace = _workspace(L.twn_ternarize_batch_workspace_bytes(len(Ws)), Ws[0].device)
    fn = L.twn_ternarize_batch
    args = (items, len(Ws), ctypes.c_float(delta_factor), _ptr(workspace), workspace.numel())
    keep = (items, list(Ws), list(out), workspace)

    def call(stream=None, _keep=keep):
        rc = fn(*args, _stream(stream))
        if rc != 0:
            raise TwnError(rc, "twn_ternarize_batch")
        return out
    return call
