"""Thin ctypes binding over libflashd.so: argument marshalling only.

Function names mirror the C ABI in include/flashd.h.  Tensors are torch CUDA
(ROCm) tensors used purely as owners of device memory; every step of the
computation runs inside the library's HIP kernels.  There is no fallback: if the
shared library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflashd.so")

F32, F16, BF16 = 0, 1, 2
VARIANT_AUTO, VARIANT_TILE, VARIANT_PER_KEY, VARIANT_ONLINE_SOFTMAX, VARIANT_TILE_BLEND = 0, 1, 2, 3, 4
VARIANT_TILE_256 = 5
MAX_SPLITS = 64
STATIC_SCRATCH_BYTES = 32 << 20

_DTYPE = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}

EXPORTS = ("flashd_attn_fwd", "flashd_attn_fwd_ex", "flashd_workspace_bytes",
           "flashd_auto_splits", "flashd_auto_variant", "flashd_status_string", "flashd_version", "flashd_skip_stats", "flashd_attn_fwd_state",
           "flashd_attn_fwd_kv8", "flashd_attn_fwd_static", "flashd_attn_fwd_skipv",
           "flashd_release_workspace")


class FlashdError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"libflashd status {status}: {status_string(status)}")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2505_14201_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i, f, p, z = ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
    base = [p, p, p, p, i, i, i, i, i, i, i, f, i, p]
    lib.flashd_attn_fwd.restype = i
    lib.flashd_attn_fwd.argtypes = base
    lib.flashd_attn_fwd_static.restype = i
    lib.flashd_attn_fwd_static.argtypes = base
    lib.flashd_attn_fwd_ex.restype = i
    lib.flashd_attn_fwd_skipv.restype = i
    lib.flashd_attn_fwd_skipv.argtypes = base + [i, p, z, p]
    lib.flashd_attn_fwd_ex.argtypes = base + [i, i, p, z]
    lib.flashd_workspace_bytes.restype = z
    lib.flashd_workspace_bytes.argtypes = [i] * 9
    lib.flashd_auto_splits.restype = i
    lib.flashd_auto_splits.argtypes = [i] * 8
    lib.flashd_auto_variant.restype = i
    lib.flashd_auto_variant.argtypes = [i] * 8
    lib.flashd_attn_fwd_state.restype = i
    lib.flashd_attn_fwd_state.argtypes = [p, p, p, p, p, p, i, i, i, i, i, i, i, i, f, i, p]
    lib.flashd_attn_fwd_kv8.restype = i
    lib.flashd_attn_fwd_kv8.argtypes = [p, p, p, p, i, i, i, i, i, i, i, f, f, f, i, p]
    lib.flashd_skip_stats.restype = i
    lib.flashd_skip_stats.argtypes = [p, p, i, i, i, i, i, i, i, f, i, f, f, p, p]
    lib.flashd_release_workspace.restype = i
    lib.flashd_release_workspace.argtypes = []
    lib.flashd_status_string.restype = ctypes.c_char_p
    lib.flashd_status_string.argtypes = [i]
    lib.flashd_version.restype = i
    lib.flashd_version.argtypes = []
    return lib


_lib = _load()


def raw() -> ctypes.CDLL:
    """The loaded C library (for tests that call the ABI with hand-made arguments)."""
    return _lib


def status_string(status: int) -> str:
    return _lib.flashd_status_string(int(status)).decode()


def version() -> int:
    return int(_lib.flashd_version())


def release_workspace() -> None:
    """flashd_release_workspace: free the scratch memory cached for the current device."""
    rc = int(_lib.flashd_release_workspace())
    if rc != 0:
        raise FlashdError(rc)


def workspace_bytes(B, Hq, Hkv, Lq, Lk, d, dtype, variant=VARIANT_AUTO, splits=0) -> int:
    return int(_lib.flashd_workspace_bytes(B, Hq, Hkv, Lq, Lk, d, dtype, variant, splits))


def auto_splits(B, Hq, Hkv, Lq, Lk, d, dtype, variant=VARIANT_AUTO) -> int:
    return int(_lib.flashd_auto_splits(B, Hq, Hkv, Lq, Lk, d, dtype, variant))


def auto_variant(B, Hq, Hkv, Lq, Lk, d, dtype, causal) -> int:
    return int(_lib.flashd_auto_variant(B, Hq, Hkv, Lq, Lk, d, dtype, int(bool(causal))))


def _marshal(q, k, v, o):
    for name, t in (("q", q), ("k", k), ("v", v), ("o", o)):
        if not t.is_cuda:
            raise ValueError(f"{name} must live on the GPU")
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    if q.dtype not in _DTYPE or not (k.dtype == v.dtype == o.dtype == q.dtype):
        raise ValueError("q, k, v, o must share one of float32/float16/bfloat16")
    if q.dim() != 4 or k.dim() != 4 or v.shape != k.shape or o.shape != q.shape:
        raise ValueError("expected q,o: [B,Hq,Lq,d] and k,v: [B,Hkv,Lk,d]")
    B, Hq, Lq, d = q.shape
    Bk, Hkv, Lk, dk = k.shape
    if Bk != B or dk != d:
        raise ValueError("batch or head dimension mismatch between q and k")
    return B, Hq, Hkv, Lq, Lk, d, _DTYPE[q.dtype]


def _stream_ptr(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def attn_fwd(q, k, v, o, causal: bool, scale: float, stream=None) -> None:
    """flashd_attn_fwd: o <- attention(q, k, v), enqueued on `stream` (default: current)."""
    B, Hq, Hkv, Lq, Lk, d, dt = _marshal(q, k, v, o)
    with torch.cuda.device(q.device):
        st = _stream_ptr(stream)
        rc = _lib.flashd_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                  B, Hq, Hkv, Lq, Lk, d, int(bool(causal)), float(scale), dt, st)
    if rc != 0:
        raise FlashdError(rc)


def attn_fwd_static(q, k, v, o, causal: bool, scale: float, stream=None) -> None:
    """flashd_attn_fwd_static: as attn_fwd, split-K scratch in the library's fixed array
    (no allocation; raises FlashdError(E_WORKSPACE) when the problem needs more)."""
    B, Hq, Hkv, Lq, Lk, d, dt = _marshal(q, k, v, o)
    with torch.cuda.device(q.device):
        st = _stream_ptr(stream)
        rc = _lib.flashd_attn_fwd_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                         B, Hq, Hkv, Lq, Lk, d, int(bool(causal)), float(scale),
                                         dt, st)
    if rc != 0:
        raise FlashdError(rc)


def attn_fwd_ex(q, k, v, o, causal: bool, scale: float, variant: int = VARIANT_AUTO,
                splits: int = 0, workspace=None, stream=None) -> None:
    """flashd_attn_fwd_ex: explicit variant/splits and a caller-owned workspace tensor
    (any dtype, contiguous, on the same device) of at least workspace_bytes(...) bytes."""
    B, Hq, Hkv, Lq, Lk, d, dt = _marshal(q, k, v, o)
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        if not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous GPU tensor")
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    with torch.cuda.device(q.device):
        st = _stream_ptr(stream)
        rc = _lib.flashd_attn_fwd_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                     B, Hq, Hkv, Lq, Lk, d, int(bool(causal)), float(scale), dt,
                                     st, int(variant), int(splits), ws_ptr, ws_bytes)
    if rc != 0:
        raise FlashdError(rc)


def attn_fwd_skipv(q, k, v, o, causal: bool, scale: float, splits: int = 0, workspace=None,
                   counts=None, stream=None) -> None:
    """flashd_attn_fwd_skipv: decode with the saturation skip on the V fetch.  `counts`:
    optional GPU int64 tensor of 2 elements that the launch adds (blocks visited, blocks whose
    V was not fetched) to."""
    B, Hq, Hkv, Lq, Lk, d, dt = _marshal(q, k, v, o)
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        if not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous GPU tensor")
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    if counts is not None and not (counts.is_cuda and counts.dtype == torch.int64
                                   and counts.numel() >= 2 and counts.is_contiguous()):
        raise ValueError("counts must be a contiguous GPU int64 tensor of 2 elements")
    with torch.cuda.device(q.device):
        rc = _lib.flashd_attn_fwd_skipv(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                        B, Hq, Hkv, Lq, Lk, d, int(bool(causal)), float(scale),
                                        dt, _stream_ptr(stream), int(splits), ws_ptr, ws_bytes,
                                        None if counts is None else counts.data_ptr())
    if rc != 0:
        raise FlashdError(rc)


def skip_stats(q, k, causal: bool, scale: float, lo: float = -6.0, hi: float = 11.0,
               counts=None, stream=None):
    """flashd_skip_stats: (steps, low, high) of the static skip rule.  `counts`: optional
    GPU int64 tensor of 3 elements to receive the result (then nothing is read back and the
    call only enqueues work); otherwise a tensor is created and the counts are returned."""
    if not (q.is_cuda and k.is_cuda and q.is_contiguous() and k.is_contiguous()):
        raise ValueError("q and k must be contiguous GPU tensors")
    if q.dtype not in _DTYPE or k.dtype != q.dtype or q.dim() != 4 or k.dim() != 4:
        raise ValueError("expected q: [B,Hq,Lq,d] and k: [B,Hkv,Lk,d] of one storage type")
    B, Hq, Lq, d = q.shape
    Bk, Hkv, Lk, dk = k.shape
    if Bk != B or dk != d:
        raise ValueError("batch or head dimension mismatch between q and k")
    own = counts is None
    with torch.cuda.device(q.device):
        if own:
            counts = torch.empty(3, dtype=torch.int64, device=q.device)
        elif not (counts.is_cuda and counts.dtype == torch.int64 and counts.numel() >= 3
                  and counts.is_contiguous()):
            raise ValueError("counts must be a contiguous GPU int64 tensor of 3 elements")
        rc = _lib.flashd_skip_stats(q.data_ptr(), k.data_ptr(), B, Hq, Hkv, Lq, Lk, d,
                                    int(bool(causal)), float(scale), _DTYPE[q.dtype], float(lo),
                                    float(hi), counts.data_ptr(), _stream_ptr(stream))
    if rc != 0:
        raise FlashdError(rc)
    if not own:
        return None
    c = counts.cpu()
    return int(c[0]), int(c[1]), int(c[2])


def attn_fwd_state(q, k, v, causal: bool, scale: float, o=None, state_in=None, state_out=None,
                   causal_shift=None, stream=None) -> None:
    """flashd_attn_fwd_state: one chunk of keys with the Alg. 3 state handed in and out.
    States are float32 GPU tensors [B, Hq, Lq, d + 2]; causal_shift defaults to Lk - Lq."""
    for name, t in (("q", q), ("k", k), ("v", v)):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous GPU tensor")
    if q.dtype not in _DTYPE or not (k.dtype == v.dtype == q.dtype):
        raise ValueError("q, k, v must share one of float32/float16/bfloat16")
    B, Hq, Lq, d = q.shape
    Bk, Hkv, Lk, dk = k.shape
    if Bk != B or dk != d or v.shape != k.shape:
        raise ValueError("shape mismatch between q, k and v")
    if o is not None and (o.shape != q.shape or o.dtype != q.dtype or not o.is_cuda
                          or not o.is_contiguous()):
        raise ValueError("o must match q")
    for name, t in (("state_in", state_in), ("state_out", state_out)):
        if t is not None and (tuple(t.shape) != (B, Hq, Lq, d + 2) or t.dtype != torch.float32
                              or not t.is_cuda or not t.is_contiguous()):
            raise ValueError(f"{name} must be a contiguous float32 GPU tensor [B, Hq, Lq, d + 2]")
    shift = Lk - Lq if causal_shift is None else int(causal_shift)
    ptr = lambda t: None if t is None else t.data_ptr()
    with torch.cuda.device(q.device):
        rc = _lib.flashd_attn_fwd_state(q.data_ptr(), k.data_ptr(), v.data_ptr(), ptr(o),
                                        ptr(state_in), ptr(state_out), B, Hq, Hkv, Lq, Lk, d,
                                        int(bool(causal)), shift, float(scale), _DTYPE[q.dtype],
                                        _stream_ptr(stream))
    if rc != 0:
        raise FlashdError(rc)


def attn_fwd_kv8(q, k8, v8, o, causal: bool, scale: float, kscale: float, vscale: float,
                 stream=None) -> None:
    """flashd_attn_fwd_kv8: K and V as torch.float8_e4m3fn tensors [B, Hkv, Lk, d] (the real
    values are kscale * k8 and vscale * v8); q and o float16 or bfloat16."""
    for name, t in (("q", q), ("k8", k8), ("v8", v8), ("o", o)):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous GPU tensor")
    if q.dtype not in (torch.float16, torch.bfloat16) or o.dtype != q.dtype or o.shape != q.shape:
        raise ValueError("q and o must be float16 or bfloat16 tensors of one shape")
    if k8.dtype != torch.float8_e4m3fn or v8.dtype != k8.dtype or v8.shape != k8.shape:
        raise ValueError("k8 and v8 must be float8_e4m3fn tensors of one shape")
    B, Hq, Lq, d = q.shape
    Bk, Hkv, Lk, dk = k8.shape
    if Bk != B or dk != d:
        raise ValueError("batch or head dimension mismatch between q and k8")
    with torch.cuda.device(q.device):
        rc = _lib.flashd_attn_fwd_kv8(q.data_ptr(), k8.data_ptr(), v8.data_ptr(), o.data_ptr(),
                                      B, Hq, Hkv, Lq, Lk, d, int(bool(causal)), float(scale),
                                      float(kscale), float(vscale), _DTYPE[q.dtype],
                                      _stream_ptr(stream))
    if rc != 0:
        raise FlashdError(rc)
