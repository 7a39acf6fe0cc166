"""Thin Python binding of libbra (BRA forward on MI355X): argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/bra.h.  torch is used for device memory and the current stream.  There is
no CPU fallback: if libbra.so has not been built, importing the entry points fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbra.so")

BRA_F32, BRA_BF16 = 0, 1
PATH_AUTO, PATH_GENERIC, PATH_MFMA = 0, 1, 2
_PATHS = {"auto": PATH_AUTO, "generic": PATH_GENERIC, "mfma": PATH_MFMA}

STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = ("bra_workspace_bytes", "bra_route", "bra_forward", "bra_forward_static", "bra_padded_workspace_bytes",
           "bra_forward_padded", "bra_backward_workspace_bytes", "bra_backward", "bra_block_workspace_bytes",
           "bra_block_forward", "bra_strerror", "bra_version",
           "bra_profile_begin", "bra_profile_end", "bra_kernel_name", "bra_util_copy",
           "bra_util_read", "bra_util_mfma", "bra_util_mfma32")


class BraShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("C", ctypes.c_int32), ("heads", ctypes.c_int32), ("S", ctypes.c_int32),
                ("k", ctypes.c_int32), ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
                ("path", ctypes.c_int32)]


class BraBlockParams(ctypes.Structure):
    """bra_block_params: device pointers, in the order of include/bra.h."""
    FIELDS = ("Wpos", "bpos", "ln1_g", "ln1_b", "Wqkv", "Wo", "Wlce", "ln2_g", "ln2_b", "W1", "b1", "W2", "b2")
    MATRICES = ("Wpos", "Wqkv", "Wo", "Wlce", "W1", "W2")
    _fields_ = [(name, ctypes.c_void_p) for name in FIELDS]


class BraError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libbra error {code}: {text}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libbra.so (built by paper_2303_08810_amd/build.py); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2303_08810_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        L.bra_workspace_bytes.restype = ctypes.c_int
        L.bra_workspace_bytes.argtypes = [ctypes.POINTER(BraShape), ctypes.POINTER(sz)]
        L.bra_route.restype = ctypes.c_int
        L.bra_route.argtypes = [ctypes.POINTER(BraShape), vp, vp, vp, vp, vp, sz, vp]
        L.bra_forward.restype = ctypes.c_int
        L.bra_forward.argtypes = [ctypes.POINTER(BraShape), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.bra_forward_static.restype = ctypes.c_int
        L.bra_forward_static.argtypes = [ctypes.POINTER(BraShape), vp, vp, vp, vp, vp, vp, vp, vp]
        L.bra_padded_workspace_bytes.restype = ctypes.c_int
        L.bra_padded_workspace_bytes.argtypes = [ctypes.POINTER(BraShape), ctypes.POINTER(sz)]
        L.bra_forward_padded.restype = ctypes.c_int
        L.bra_forward_padded.argtypes = [ctypes.POINTER(BraShape), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.bra_backward_workspace_bytes.restype = ctypes.c_int
        L.bra_backward_workspace_bytes.argtypes = [ctypes.POINTER(BraShape), ctypes.POINTER(sz)]
        L.bra_backward.restype = ctypes.c_int
        L.bra_backward.argtypes = [ctypes.POINTER(BraShape)] + [vp] * 11 + [sz, vp]
        L.bra_block_workspace_bytes.restype = ctypes.c_int
        L.bra_block_workspace_bytes.argtypes = [ctypes.POINTER(BraShape), ctypes.c_int32, ctypes.POINTER(sz)]
        L.bra_block_forward.restype = ctypes.c_int
        L.bra_block_forward.argtypes = [ctypes.POINTER(BraShape), ctypes.c_int32, ctypes.c_float, vp,
                                        ctypes.POINTER(BraBlockParams), vp, vp, vp, vp, sz, vp]
        L.bra_strerror.restype = ctypes.c_char_p
        L.bra_strerror.argtypes = [ctypes.c_int]
        L.bra_version.restype = ctypes.c_int
        L.bra_version.argtypes = []
        L.bra_profile_begin.restype = ctypes.c_int
        L.bra_profile_begin.argtypes = [ctypes.c_int]
        L.bra_profile_end.restype = ctypes.c_int
        L.bra_profile_end.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float),
                                      ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        L.bra_kernel_name.restype = ctypes.c_char_p
        L.bra_kernel_name.argtypes = [ctypes.c_int]
        L.bra_util_copy.restype = ctypes.c_int
        L.bra_util_copy.argtypes = [vp, vp, sz, vp]
        L.bra_util_read.restype = ctypes.c_int
        L.bra_util_read.argtypes = [vp, sz, vp, vp]
        L.bra_util_mfma.restype = ctypes.c_int
        L.bra_util_mfma.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp]
        L.bra_util_mfma32.restype = ctypes.c_int
        L.bra_util_mfma32.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().bra_strerror(int(code)).decode()


def _check(code: int) -> None:
    if code != 0:
        raise BraError(code, strerror(code))


def make_shape(B, H, W, C, heads, S, k, dtype, scale=None, path="auto") -> BraShape:
    dt = {torch.float32: BRA_F32, torch.bfloat16: BRA_BF16}.get(dtype, dtype)
    return BraShape(B, H, W, C, heads, S, k, int(dt), float(scale) if scale else 0.0, _PATHS[path])


def workspace_bytes(shape: BraShape) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().bra_workspace_bytes(ctypes.byref(shape), ctypes.byref(out)))
    return out.value


def alloc_workspace(shape: BraShape, device) -> torch.Tensor:
    nbytes = max(workspace_bytes(shape), 256)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    assert ws.data_ptr() % 256 == 0
    return ws


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _stream(device) -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def _check_inputs(X, Wqkv, Wo=None, Wlce=None):
    B, H, W, C = X.shape
    for t in (X, Wqkv, Wo, Wlce):
        if t is None:
            continue
        if not (t.is_cuda and t.is_contiguous() and t.dtype == X.dtype and t.device == X.device):
            raise ValueError("tensors must be contiguous, on one GPU and of one dtype")
    if tuple(Wqkv.shape) != (C, 3 * C):
        raise ValueError("Wqkv must be [C, 3C]")
    if Wo is not None and tuple(Wo.shape) != (C, C):
        raise ValueError("Wo must be [C, C]")
    if Wlce is not None and tuple(Wlce.shape) != (C, 5, 5):
        raise ValueError("Wlce must be [C, 5, 5]")
    return B, H, W, C


def bra_route(X, Wqkv, S, k, heads, *, want_Ar=False, path="auto", ws=None):
    """Routing index I^r [B, S*S, k] (int32) and, optionally, A^r [B, S*S, S*S] (float32)."""
    B, H, W, C = _check_inputs(X, Wqkv)
    shape = make_shape(B, H, W, C, heads, S, k, X.dtype, None, path)
    if ws is None:
        ws = alloc_workspace(shape, X.device)
    Ir = torch.empty((B, S * S, k), dtype=torch.int32, device=X.device)
    Ar = torch.empty((B, S * S, S * S), dtype=torch.float32, device=X.device) if want_Ar else None
    _check(lib().bra_route(ctypes.byref(shape), _ptr(X), _ptr(Wqkv), _ptr(Ir), _ptr(Ar), _ptr(ws),
                           ws.numel(), _stream(X.device)))
    return (Ir, Ar) if want_Ar else Ir


def bra_forward(X, Wqkv, Wo, Wlce, S, k, heads, *, scale=None, Ir_in=None, want_Ir=False,
                path="auto", ws=None, out=None):
    """Y [B, H, W, C] = BRA(X); optionally also the routing index that was used."""
    B, H, W, C = _check_inputs(X, Wqkv, Wo, Wlce)
    shape = make_shape(B, H, W, C, heads, S, k, X.dtype, scale, path)
    if ws is None:
        ws = alloc_workspace(shape, X.device)
    Y = out if out is not None else torch.empty_like(X)
    Ir = torch.empty((B, S * S, k), dtype=torch.int32, device=X.device) if want_Ir else None
    if Ir_in is not None:
        if not (Ir_in.is_cuda and Ir_in.is_contiguous() and Ir_in.dtype == torch.int32
                and tuple(Ir_in.shape) == (B, S * S, k)):
            raise ValueError("Ir_in must be a contiguous int32 [B, S*S, k] device tensor")
    _check(lib().bra_forward(ctypes.byref(shape), _ptr(X), _ptr(Wqkv), _ptr(Wo), _ptr(Wlce), _ptr(Y),
                             _ptr(Ir), _ptr(Ir_in), _ptr(ws), ws.numel(), _stream(X.device)))
    return (Y, Ir) if want_Ir else Y


def bra_forward_static(X, Wqkv, Wo, Wlce, S, k, heads, *, out, Ir_out=None, Ir_in=None, scale=None, path="auto"):
    """bra_forward on the library's built-in scratch buffer: nothing is allocated, here or in the
    library.  `out` [B, H, W, C] and, if wanted, `Ir_out` [B, S*S, k] (int32) are the caller's."""
    B, H, W, C = _check_inputs(X, Wqkv, Wo, Wlce)
    shape = make_shape(B, H, W, C, heads, S, k, X.dtype, scale, path)
    for t, shp, dt in ((out, (B, H, W, C), X.dtype), (Ir_out, (B, S * S, k), torch.int32), (Ir_in, (B, S * S, k), torch.int32)):
        if t is not None and not (t.is_cuda and t.is_contiguous() and t.dtype == dt and tuple(t.shape) == shp):
            raise ValueError(f"expected a contiguous {dt} device tensor of shape {shp}")
    _check(lib().bra_forward_static(ctypes.byref(shape), _ptr(X), _ptr(Wqkv), _ptr(Wo), _ptr(Wlce), _ptr(out),
                                    _ptr(Ir_out), _ptr(Ir_in), _stream(X.device)))
    return out


def bra_forward_padded(X, Wqkv, Wo, Wlce, S, k, heads, *, scale=None, Ir_in=None, want_Ir=False, path="auto"):
    """BRA on a map whose sides S need not divide: zero tokens are appended at the bottom and right,
    Y is the top-left H x W part of the result (see include/bra.h)."""
    B, H, W, C = _check_inputs(X, Wqkv, Wo, Wlce)
    shape = make_shape(B, H, W, C, heads, S, k, X.dtype, scale, path)
    need = ctypes.c_size_t(0)
    _check(lib().bra_padded_workspace_bytes(ctypes.byref(shape), ctypes.byref(need)))
    ws = torch.empty(max(need.value, 256), dtype=torch.uint8, device=X.device)
    Y = torch.empty_like(X)
    Ir = torch.empty((B, S * S, k), dtype=torch.int32, device=X.device) if want_Ir else None
    if Ir_in is not None:
        if not (Ir_in.is_cuda and Ir_in.is_contiguous() and Ir_in.dtype == torch.int32
                and tuple(Ir_in.shape) == (B, S * S, k)):
            raise ValueError("Ir_in must be a contiguous int32 [B, S*S, k] device tensor")
    _check(lib().bra_forward_padded(ctypes.byref(shape), _ptr(X), _ptr(Wqkv), _ptr(Wo), _ptr(Wlce), _ptr(Y),
                                    _ptr(Ir), _ptr(Ir_in), _ptr(ws), ws.numel(), _stream(X.device)))
    return (Y, Ir) if want_Ir else Y


def bra_backward(X, Wqkv, Wo, Wlce, Ir, dY, S, heads, *, scale=None, path="auto", ws=None):
    """Gradients of the layer for fixed routing Ir [B, S*S, k] (see include/bra.h): returns
    (dX in X's dtype, dWqkv, dWo, dWlce in float32).  path: "auto", "generic" (scalar float32
    kernels) or "mfma" (matrix-core kernels; raises if the shape is outside their range)."""
    B, H, W, C = _check_inputs(X, Wqkv, Wo, Wlce)
    k = int(Ir.shape[-1])
    if not (Ir.is_cuda and Ir.is_contiguous() and Ir.dtype == torch.int32 and tuple(Ir.shape) == (B, S * S, k)):
        raise ValueError("Ir must be a contiguous int32 [B, S*S, k] device tensor")
    if not (dY.is_cuda and dY.is_contiguous() and dY.dtype == X.dtype and dY.shape == X.shape):
        raise ValueError("dY must match X")
    shape = make_shape(B, H, W, C, heads, S, k, X.dtype, scale, path)
    if ws is None:
        need = ctypes.c_size_t(0)
        _check(lib().bra_backward_workspace_bytes(ctypes.byref(shape), ctypes.byref(need)))
        ws = torch.empty(max(need.value, 256), dtype=torch.uint8, device=X.device)
    dX = torch.empty_like(X)
    dWqkv = torch.empty((C, 3 * C), dtype=torch.float32, device=X.device)
    dWo = torch.empty((C, C), dtype=torch.float32, device=X.device)
    dWlce = torch.empty((C, 5, 5), dtype=torch.float32, device=X.device)
    _check(lib().bra_backward(ctypes.byref(shape), _ptr(X), _ptr(Wqkv), _ptr(Wo), _ptr(Wlce), _ptr(Ir), _ptr(dY),
                              _ptr(dX), _ptr(dWqkv), _ptr(dWo), _ptr(dWlce), _ptr(ws), ws.numel(), _stream(X.device)))
    return dX, dWqkv, dWo, dWlce


def block_workspace_bytes(shape: BraShape, hidden: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().bra_block_workspace_bytes(ctypes.byref(shape), int(hidden), ctypes.byref(out)))
    return out.value


def bra_block_forward(X, params, S, k, heads, *, eps=1e-6, scale=None, Ir_in=None, want_Ir=False,
                      path="auto", ws=None, out=None):
    """One whole BiFormer block (position encoding, LayerNorm, BRA, LayerNorm, MLP with residual
    links; see include/bra.h).  `params`: dict of device tensors named as BraBlockParams.FIELDS;
    the matrices in X's dtype, the vectors float32."""
    B, H, W, C = X.shape
    hidden = int(params["W1"].shape[1])
    want = {"Wpos": (C, 3, 3), "bpos": (C,), "ln1_g": (C,), "ln1_b": (C,), "Wqkv": (C, 3 * C), "Wo": (C, C),
            "Wlce": (C, 5, 5), "ln2_g": (C,), "ln2_b": (C,), "W1": (C, hidden), "b1": (hidden,),
            "W2": (hidden, C), "b2": (C,)}
    if not (X.is_cuda and X.is_contiguous()):
        raise ValueError("X must be a contiguous device tensor")
    for name in BraBlockParams.FIELDS:
        t = params[name]
        dt = X.dtype if name in BraBlockParams.MATRICES else torch.float32
        if not (t.is_cuda and t.is_contiguous() and t.device == X.device and t.dtype == dt
                and tuple(t.shape) == want[name]):
            raise ValueError(f"{name} must be a contiguous {dt} device tensor of shape {want[name]}")
    shape = make_shape(B, H, W, C, heads, S, k, X.dtype, scale, path)
    if ws is None:
        ws = torch.empty(max(block_workspace_bytes(shape, hidden), 256), dtype=torch.uint8, device=X.device)
        assert ws.data_ptr() % 256 == 0
    Xout = out if out is not None else torch.empty_like(X)
    Ir = torch.empty((B, S * S, k), dtype=torch.int32, device=X.device) if want_Ir else None
    if Ir_in is not None:
        if not (Ir_in.is_cuda and Ir_in.is_contiguous() and Ir_in.dtype == torch.int32
                and tuple(Ir_in.shape) == (B, S * S, k)):
            raise ValueError("Ir_in must be a contiguous int32 [B, S*S, k] device tensor")
    P = BraBlockParams(*[params[name].data_ptr() for name in BraBlockParams.FIELDS])
    _check(lib().bra_block_forward(ctypes.byref(shape), hidden, float(eps), _ptr(X), ctypes.byref(P), _ptr(Xout),
                                   _ptr(Ir), _ptr(Ir_in), _ptr(ws), ws.numel(), _stream(X.device)))
    return (Xout, Ir) if want_Ir else Xout


def profile_begin(max_records: int) -> None:
    """Start per-launch timing of the library's kernels (see include/bra.h)."""
    _check(lib().bra_profile_begin(int(max_records)))


def profile_end(max_records: int):
    """Stop per-launch timing; returns [(kernel name, milliseconds), ...] in launch order."""
    ids = (ctypes.c_int32 * max_records)()
    ms = (ctypes.c_float * max_records)()
    n = ctypes.c_int(0)
    _check(lib().bra_profile_end(ids, ms, max_records, ctypes.byref(n)))
    return [(lib().bra_kernel_name(ids[i]).decode(), float(ms[i])) for i in range(n.value)]


def util_mfma(workgroups: int, iters: int, scratch: torch.Tensor) -> None:
    """Matrix-core throughput probe: workgroups x 4 wavefronts x 8 iters dense bf16 16x16x32 products."""
    _check(lib().bra_util_mfma(int(workgroups), int(iters), _ptr(scratch), _stream(scratch.device)))


def util_mfma32(workgroups: int, iters: int, scratch: torch.Tensor) -> None:
    """Matrix-core throughput probe: workgroups x 4 wavefronts x 4 iters dense bf16 32x32x16 products."""
    _check(lib().bra_util_mfma32(int(workgroups), int(iters), _ptr(scratch), _stream(scratch.device)))


def util_read(src: torch.Tensor, scratch: torch.Tensor) -> None:
    """Plain read-only pass over src, for bandwidth calibration."""
    _check(lib().bra_util_read(_ptr(src), src.numel() * src.element_size(), _ptr(scratch), _stream(src.device)))


def util_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Plain device copy of src into dst (same byte size), for bandwidth calibration."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().bra_util_copy(_ptr(dst), _ptr(src), nbytes, _stream(src.device)))
