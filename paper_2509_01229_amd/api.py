"""Thin Python binding of the C ABI in include/liquidgemm.h (argument marshalling only).

Host entry points take and return numpy arrays; device entry points take torch tensors
that live on the GPU (torch is used for device memory and streams, nothing else) and
enqueue on torch's current stream unless `stream` (a raw hipStream_t integer) is given.
Every step of the path runs inside libliquidgemm.so; if the library has not been built
the first call raises -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# LIQUIDGEMM_LIB lets tools load another build of the same library (e.g. an experiment build)
LIB_PATH = os.environ.get("LIQUIDGEMM_LIB") or os.path.join(_PKG, "libliquidgemm.so")
_lib = None

LQ_OK = 0
LQ_ERR_INVALID, LQ_ERR_ALIGN, LQ_ERR_WORKSPACE, LQ_ERR_HIP = -1, -2, -3, -4


class LiquidGemmError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"liquidgemm error {code}: {message}")
        self.code = code


def lib() -> ctypes.CDLL:
    """Load libliquidgemm.so (built by `python -m paper_2509_01229_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2509_01229_amd.build` "
            "(there is no CPU fallback for the GEMM path)")
    # torch ships its own HIP runtime; load it first so that the library binds to the
    # same runtime that owns the device pointers and streams it is handed.
    import torch  # noqa: F401

    L = ctypes.CDLL(LIB_PATH)
    i, vp, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    L.w4a8_version.restype = i
    L.w4a8_last_error.restype = ctypes.c_char_p
    L.liquidquant_packed_size.restype = i
    L.liquidquant_packed_size.argtypes = [i, i, i, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.liquidquant_pack_weights.restype = i
    L.liquidquant_pack_weights.argtypes = [vp, i, i, i, vp, vp, vp]
    L.liquidquant_pack_weights_f16.restype = i
    L.liquidquant_pack_weights_f16.argtypes = [vp, i, i, i, vp, vp, vp]
    L.liquidquant_pack_from_i8.restype = i
    L.liquidquant_pack_from_i8.argtypes = [vp, i, i, i, vp, vp]
    L.liquidquant_unpack_weights.restype = i
    L.liquidquant_unpack_weights.argtypes = [vp, vp, i, i, i, vp, vp, vp]
    L.w4a8_gemm_workspace_size.restype = sz
    L.w4a8_gemm_workspace_size.argtypes = [i, i, i, i]
    L.w4a8_workspace_init.restype = i
    L.w4a8_workspace_init.argtypes = [vp, sz, vp]
    L.w4a8_gemm.restype = i
    L.w4a8_gemm.argtypes = [i, i, i, i, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.w4a8_gemm_static.restype = i
    L.w4a8_gemm_static.argtypes = [i, i, i, i, vp, vp, vp, vp, vp, vp, vp]
    L.w4a8_gemm_i32.restype = i
    L.w4a8_gemm_i32.argtypes = [i, i, i, i, vp, vp, vp, vp, vp, sz, vp]
    L.w4a8_gemm_variant.restype = i
    L.w4a8_gemm_variant.argtypes = [i, i, i, i, i, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.w4a8_variant_count.restype = i
    L.w4a8_variant_name.restype = ctypes.c_char_p
    L.w4a8_variant_name.argtypes = [i]
    L.w4a8_variant_supports.restype = i
    L.w4a8_variant_supports.argtypes = [i, i, i, i, i]
    L.w4a8_select_variant.restype = i
    L.w4a8_select_variant.argtypes = [i, i, i, i]
    L.w4a8_select_plan.restype = i
    L.w4a8_select_plan.argtypes = [i, i, i, i, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    L.w4a8_dequant_dump.restype = i
    L.w4a8_dequant_dump.argtypes = [vp, vp, i, i, i, vp, vp]
    L.w4a8_grouped_gemm.restype = i
    L.w4a8_grouped_gemm.argtypes = [i, ctypes.POINTER(ctypes.c_int), i, i, i, vp, vp, vp, vp, vp, vp, vp, vp]
    L.w4a8_quantize_activations.restype = i
    L.w4a8_quantize_activations.argtypes = [i, i, vp, vp, vp, vp, vp]
    L.w8a8_pack_weights.restype = i
    L.w8a8_pack_weights.argtypes = [vp, i, i, vp]
    L.w8a8_gemm.restype = i
    L.w8a8_gemm.argtypes = [i, i, i, vp, vp, vp, vp, vp, vp, vp]
    L.w4a8_calib_stream_read.restype = i
    L.w4a8_calib_stream_read.argtypes = [vp, sz, vp]
    L.w4a8_calib_mfma_i8.restype = i
    L.w4a8_calib_mfma_i8.argtypes = [i, i, ctypes.POINTER(ctypes.c_double), vp]
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != LQ_OK:
        raise LiquidGemmError(rc, lib().w4a8_last_error().decode())


def _np(a):
    return a.ctypes.data_as(ctypes.c_void_p)


# ----------------------------------------------------------------------------- host side
def w4a8_version() -> int:
    return int(lib().w4a8_version())


def liquidquant_packed_size(N: int, K: int, group: int):
    cb, gb = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().liquidquant_packed_size(N, K, group, ctypes.byref(cb), ctypes.byref(gb)))
    return int(cb.value), int(gb.value)


def _alloc_packed(N, K, group):
    cb, gb = liquidquant_packed_size(N, K, group)
    return np.empty(cb, dtype=np.uint8), np.empty(gb, dtype=np.uint8)


def liquidquant_pack_weights(W, group: int):
    """W: numpy [N,K] float32 (FP16-valued) or float16.  Returns (W_packed, gparams, w_scales)."""
    W = np.ascontiguousarray(W)
    if W.ndim != 2:
        raise ValueError("W must be [N, K]")
    N, K = W.shape
    packed, gparams = _alloc_packed(N, K, group)
    w_scales = np.empty(N, dtype=np.float32)
    if W.dtype == np.float16:
        rc = lib().liquidquant_pack_weights_f16(_np(W.view(np.uint16)), N, K, group, _np(packed),
                                                _np(gparams), _np(w_scales))
    elif W.dtype == np.float32:
        rc = lib().liquidquant_pack_weights(_np(W), N, K, group, _np(packed), _np(gparams), _np(w_scales))
    else:
        raise TypeError("W must be float32 or float16")
    _check(rc)
    return packed, gparams, w_scales


def liquidquant_pack_from_i8(Q_i8, group: int):
    Q = np.ascontiguousarray(Q_i8, dtype=np.int8)
    N, K = Q.shape
    packed, gparams = _alloc_packed(N, K, group)
    _check(lib().liquidquant_pack_from_i8(_np(Q), N, K, group, _np(packed), _np(gparams)))
    return packed, gparams


def w8a8_pack_weights(W_i8):
    """INT8 weights [N,K] (numpy) in the order the W8A8 reference kernel consumes them: uint8 [N*K]."""
    W = np.ascontiguousarray(W_i8, dtype=np.int8)
    if W.ndim != 2:
        raise ValueError("W must be [N, K]")
    N, K = W.shape
    packed = np.empty(N * K, dtype=np.uint8)
    _check(lib().w8a8_pack_weights(_np(W), N, K, _np(packed)))
    return packed


def liquidquant_unpack_weights(W_packed, gparams, N: int, K: int, group: int):
    """Returns (codes [N,K] uint8, s_u8 [N,K/group] uint8, a [N,K/group] uint8)."""
    W_packed = np.ascontiguousarray(W_packed, dtype=np.uint8)
    gparams = np.ascontiguousarray(gparams, dtype=np.uint8)
    cb, gb = liquidquant_packed_size(N, K, group)
    if W_packed.size != cb or gparams.size != gb:
        raise ValueError("packed blob has the wrong size for this shape")
    codes = np.empty((N, K), dtype=np.uint8)
    s_u8 = np.empty((N, K // group), dtype=np.uint8)
    a = np.empty((N, K // group), dtype=np.uint8)
    _check(lib().liquidquant_unpack_weights(_np(W_packed), _np(gparams), N, K, group, _np(codes),
                                            _np(s_u8), _np(a)))
    return codes, s_u8, a


# --------------------------------------------------------------------------- device side
def _dev(t, dtype, shape=None, name="tensor"):
    import torch

    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a torch tensor on the GPU")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch

    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(int(stream))


def w4a8_gemm_workspace_size(M: int, N: int, K: int, group: int) -> int:
    return int(lib().w4a8_gemm_workspace_size(M, N, K, group))


_ws_cache = {}
_ws_retired = []


def w4a8_workspace_init(workspace, stream=None) -> None:
    """Zero the ticket area at the head of a workspace tensor (uint8, on the GPU)."""
    import torch

    _check(lib().w4a8_workspace_init(_dev(workspace, torch.uint8, name="workspace"), workspace.numel(),
                                     _stream(stream)))


def _ws(workspace, M=0, N=0, K=0, group=64, device=None, stream=None):
    """Workspace pointer and size.  With workspace=None a zero-initialised buffer of the size
    the library asks for is allocated once per (device, stream) and reused: calls on different
    streams may overlap and must not share one (device memory plumbing, nothing else)."""
    import torch

    if workspace is None:
        if device is not None and torch.device(device).type != "cuda":
            raise TypeError("X must be a torch tensor on the GPU")
        need = w4a8_gemm_workspace_size(M, N, K, group) if M > 0 else 0
        if need == 0:
            return None, 0
        key = (str(device), int(stream) if stream is not None else int(torch.cuda.current_stream().cuda_stream))
        buf = _ws_cache.get(key)
        if buf is None or buf.numel() < need:
            # A raw stream is unknown to torch's allocator, so a superseded buffer is kept
            # alive (earlier launches on that stream may still use it) and the new one is
            # zeroed under a device-wide synchronisation before any stream can see it.
            if buf is not None:
                _ws_retired.append(buf)
            buf = torch.zeros(need, dtype=torch.uint8, device=device)
            torch.cuda.synchronize(device)
            _ws_cache[key] = buf
        workspace = buf
    return _dev(workspace, torch.uint8, name="workspace"), workspace.numel()


def w4a8_gemm(X, act_scales, W_packed, gparams, w_scales, N: int, K: int, group: int, out=None,
              workspace=None, stream=None):
    """Y [M,N] float16 = epilogue(X . dequant(W)^T); all tensors on the GPU."""
    import torch

    M = X.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    wsp, wsb = _ws(workspace, M, N, K, group, X.device, stream)
    cb, gb = liquidquant_packed_size(N, K, group)
    _check(lib().w4a8_gemm(M, N, K, group, _dev(X, torch.int8, (M, K), "X"),
                           _dev(act_scales, torch.float32, (M,), "act_scales"),
                           _dev(W_packed, torch.uint8, (cb,), "W_packed"),
                           _dev(gparams, torch.uint8, (gb,), "gparams"),
                           _dev(w_scales, torch.float32, (N,), "w_scales"),
                           _dev(out, torch.float16, (M, N), "out"), wsp, wsb, _stream(stream)))
    return out


def w4a8_gemm_static(X, act_scales, W_packed, gparams, w_scales, N: int, K: int, group: int, out, stream=None):
    """w4a8_gemm on the library's built-in split-K workspace: nothing is allocated, so `out`
    ([M,N] float16 on the GPU) must be given."""
    import torch

    M = X.shape[0]
    cb, gb = liquidquant_packed_size(N, K, group)
    _check(lib().w4a8_gemm_static(M, N, K, group, _dev(X, torch.int8, (M, K), "X"),
                                  _dev(act_scales, torch.float32, (M,), "act_scales"),
                                  _dev(W_packed, torch.uint8, (cb,), "W_packed"),
                                  _dev(gparams, torch.uint8, (gb,), "gparams"),
                                  _dev(w_scales, torch.float32, (N,), "w_scales"),
                                  _dev(out, torch.float16, (M, N), "out"), _stream(stream)))
    return out


def w4a8_gemm_i32(X, W_packed, gparams, N: int, K: int, group: int, out=None, workspace=None,
                  stream=None):
    """Raw INT32 accumulators ACC [M,N] of the same kernels."""
    import torch

    M = X.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=X.device)
    wsp, wsb = _ws(workspace, M, N, K, group, X.device, stream)
    cb, gb = liquidquant_packed_size(N, K, group)
    _check(lib().w4a8_gemm_i32(M, N, K, group, _dev(X, torch.int8, (M, K), "X"),
                               _dev(W_packed, torch.uint8, (cb,), "W_packed"),
                               _dev(gparams, torch.uint8, (gb,), "gparams"),
                               _dev(out, torch.int32, (M, N), "out"), wsp, wsb, _stream(stream)))
    return out


def w4a8_gemm_variant(variant: int, X, act_scales, W_packed, gparams, w_scales, N: int, K: int,
                      group: int, want_y=True, want_acc=True, out_y=None, out_acc=None,
                      workspace=None, stream=None):
    """Run one named kernel variant; returns (Y or None, ACC or None)."""
    import torch

    M = X.shape[0]
    if want_y and out_y is None:
        out_y = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if want_acc and out_acc is None:
        out_acc = torch.empty((M, N), dtype=torch.int32, device=X.device)
    wsp, wsb = _ws(workspace, M, N, K, group, X.device, stream)
    cb, gb = liquidquant_packed_size(N, K, group)
    _check(lib().w4a8_gemm_variant(
        variant, M, N, K, group, _dev(X, torch.int8, (M, K), "X"),
        _dev(act_scales, torch.float32, (M,), "act_scales"),
        _dev(W_packed, torch.uint8, (cb,), "W_packed"), _dev(gparams, torch.uint8, (gb,), "gparams"),
        _dev(w_scales, torch.float32, (N,), "w_scales"),
        _dev(out_y, torch.float16, (M, N), "out_y") if want_y else None,
        _dev(out_acc, torch.int32, (M, N), "out_acc") if want_acc else None, wsp, wsb, _stream(stream)))
    return (out_y if want_y else None), (out_acc if want_acc else None)


def w4a8_variant_count() -> int:
    return int(lib().w4a8_variant_count())


def w4a8_variant_name(variant: int):
    s = lib().w4a8_variant_name(variant)
    return s.decode() if s else None


def w4a8_variant_names():
    return [w4a8_variant_name(i) for i in range(w4a8_variant_count())]


def w4a8_variant_supports(variant: int, M: int, N: int, K: int, group: int) -> bool:
    return bool(lib().w4a8_variant_supports(variant, M, N, K, group))


def w4a8_select_variant(M: int, N: int, K: int, group: int) -> int:
    v = int(lib().w4a8_select_variant(M, N, K, group))
    if v < 0:
        _check(v)
    return v


def w4a8_select_plan(M: int, N: int, K: int, group: int):
    """What w4a8_gemm launches for the shape: [(rows, variant index), ...], one or two launches
    over consecutive rows."""
    rows_first, rest = ctypes.c_int(0), ctypes.c_int(-1)
    v = int(lib().w4a8_select_plan(M, N, K, group, ctypes.byref(rows_first), ctypes.byref(rest)))
    if v < 0:
        _check(v)
    plan = [(int(rows_first.value), v)]
    if rest.value >= 0:
        plan.append((M - int(rows_first.value), int(rest.value)))
    return plan


def w4a8_dequant_dump(W_packed, gparams, N: int, K: int, group: int, out=None, stream=None):
    """Wd [N,K] int8 on the GPU, produced by the kernels' own unpack + dequantisation."""
    import torch

    if out is None:
        out = torch.empty((N, K), dtype=torch.int8, device=W_packed.device)
    cb, gb = liquidquant_packed_size(N, K, group)
    _check(lib().w4a8_dequant_dump(_dev(W_packed, torch.uint8, (cb,), "W_packed"),
                                   _dev(gparams, torch.uint8, (gb,), "gparams"), N, K, group,
                                   _dev(out, torch.int8, (N, K), "out"), _stream(stream)))
    return out


def w8a8_gemm(X, act_scales, W8_packed, w_scales, N: int, K: int, want_y=True, want_acc=False, out_y=None,
              out_acc=None, stream=None):
    """The W8A8 reference GEMM (no dequantisation): returns Y [M,N] float16, raw INT32
    accumulators [M,N], or both (in that order), as asked; out_y / out_acc reuse tensors."""
    import torch

    M = int(X.shape[0])
    dx = _dev(X, torch.int8, (M, K), "X")
    dw = _dev(W8_packed, torch.uint8, (N * K,), "W8_packed")
    want_y, want_acc = want_y or out_y is not None, want_acc or out_acc is not None
    Y = (out_y if out_y is not None else torch.empty((M, N), dtype=torch.float16, device=X.device)) if want_y else None
    ACC = (out_acc if out_acc is not None
           else torch.empty((M, N), dtype=torch.int32, device=X.device)) if want_acc else None
    dsx = _dev(act_scales, torch.float32, (M,), "act_scales") if want_y else None
    dsw = _dev(w_scales, torch.float32, (N,), "w_scales") if want_y else None
    _check(lib().w8a8_gemm(M, N, K, dx, dsx, dw, dsw,
                           _dev(Y, torch.float16, (M, N), "Y") if want_y else None,
                           _dev(ACC, torch.int32, (M, N), "ACC") if want_acc else None, _stream(stream)))
    if want_y and want_acc:
        return Y, ACC
    return Y if want_y else ACC


def w4a8_calib_stream_read(buf, stream=None) -> int:
    """Enqueue one pure read of the whole uint8 device tensor `buf`; returns the bytes read."""
    import torch

    n = buf.numel() // 16 * 16
    _check(lib().w4a8_calib_stream_read(_dev(buf, torch.uint8, name="buf"), n, _stream(stream)))
    return n


def w4a8_calib_mfma_i8(iters: int, random_operands: bool, stream=None) -> float:
    """Enqueue the register-only INT8 MFMA loop; returns the operation count of the launch."""
    ops = ctypes.c_double(0.0)
    _check(lib().w4a8_calib_mfma_i8(iters, 1 if random_operands else 0, ctypes.byref(ops), _stream(stream)))
    return ops.value


def w4a8_quantize_activations(X_f16, smooth=None, out_q=None, out_scales=None, stream=None):
    """Per-token INT8 quantisation of FP16 activations [M,K] on the GPU (after dividing by
    the optional FP32 smooth scales [K]); returns (X_i8 [M,K] int8, act_scales [M] float32)."""
    import torch

    M, K = X_f16.shape
    if out_q is None:
        out_q = torch.empty((M, K), dtype=torch.int8, device=X_f16.device)
    if out_scales is None:
        out_scales = torch.empty((M,), dtype=torch.float32, device=X_f16.device)
    _check(lib().w4a8_quantize_activations(
        M, K, _dev(X_f16, torch.float16, (M, K), "X_f16"),
        _dev(smooth, torch.float32, (K,), "smooth") if smooth is not None else None,
        _dev(out_q, torch.int8, (M, K), "out_q"), _dev(out_scales, torch.float32, (M,), "out_scales"),
        _stream(stream)))
    return out_q, out_scales


def w4a8_grouped_gemm(row_offsets, X, act_scales, W_packed, gparams, w_scales, N: int, K: int, group: int,
                      want_y=True, want_acc=False, out_y=None, out_acc=None, stream=None):
    """E independent W4A8 GEMMs over disjoint runs of tokens (mixture-of-experts layers).
    row_offsets: E+1 host integers; W_packed / gparams: the experts' blobs back to back on the
    GPU; w_scales: [E, N].  Returns (Y or None, ACC or None)."""
    import torch

    offs = [int(r) for r in row_offsets]
    E = len(offs) - 1
    M = offs[-1]
    if want_y and out_y is None:
        out_y = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if want_acc and out_acc is None:
        out_acc = torch.empty((M, N), dtype=torch.int32, device=X.device)
    cb, gb = liquidquant_packed_size(N, K, group)
    c_offs = (ctypes.c_int * (E + 1))(*offs)
    _check(lib().w4a8_grouped_gemm(
        E, c_offs, N, K, group, _dev(X, torch.int8, (M, K), "X"),
        _dev(act_scales, torch.float32, (M,), "act_scales"),
        _dev(W_packed, torch.uint8, (E * cb,), "W_packed"), _dev(gparams, torch.uint8, (E * gb,), "gparams"),
        _dev(w_scales, torch.float32, (E, N), "w_scales"),
        _dev(out_y, torch.float16, (M, N), "out_y") if want_y else None,
        _dev(out_acc, torch.int32, (M, N), "out_acc") if want_acc else None, _stream(stream)))
    return (out_y if want_y else None), (out_acc if want_acc else None)
