"""ctypes binding of libllla.so -- argument marshalling only."""
from __future__ import annotations

import ctypes
import functools
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libllla.so")
_MEASURE_PATH = os.path.join(_HERE, "libllla_measure.so")
_libs = {}
_use_measure = False

PATHS = {"auto": 0, "valu": 1, "mfma": 2}
_DTYPES = {torch.float32: 0, torch.bfloat16: 1}


class LlaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = int(code)
        super().__init__("%s failed: status %d (%s)" % (where, code, status_string(code)))


class _Strides(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int64), ("head", ctypes.c_int64), ("seq", ctypes.c_int64)]


def lib_path() -> str:
    return _LIB_PATH


def measure_lib_path() -> str:
    return _MEASURE_PATH


def use_measure_library(on: bool) -> None:
    """Benchmark aid: route the calls of this module through libllla_measure.so (the same sources compiled with
    per-kernel HIP events, see include/llla_measure.h) instead of the production library."""
    global _use_measure
    _use_measure = bool(on)


def _declare(L, measure: bool):
    vp, sz, i32, f32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float
    L.llla_forward_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    L.llla_forward_workspace_bytes.restype = sz
    L.llla_decode_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    L.llla_decode_workspace_bytes.restype = sz
    fwd = [vp, vp, vp, vp, _Strides, _Strides, _Strides, _Strides, i32, i32, i32, i32, i32, i32, i32, f32, f32]
    L.llla_forward.argtypes = fwd + [vp, sz, vp]
    L.llla_forward.restype = i32
    L.llla_forward_path.argtypes = fwd + [i32, vp, sz, vp]
    L.llla_forward_path.restype = i32
    L.llla_forward_ex.argtypes = fwd[:-1] + [vp, f32, vp, vp, i32, vp, sz, vp]
    L.llla_forward_ex.restype = i32
    L.llla_forward_cg_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    L.llla_forward_cg_workspace_bytes.restype = sz
    L.llla_forward_cg.argtypes = [vp, vp, vp, vp, _Strides, _Strides, _Strides, _Strides, i32, i32, i32, i32, i32, i32,
                                  f32, f32, i32, f32, vp, vp, vp, vp, sz, vp]
    L.llla_forward_cg.restype = i32
    L.llla_backward_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    L.llla_backward_workspace_bytes.restype = sz
    L.llla_backward.argtypes = [vp, vp, vp, vp, _Strides, _Strides, _Strides, _Strides, vp, vp, vp, vp, i32, i32, i32, i32,
                                i32, f32, vp, f32, i32, vp, sz, vp]
    L.llla_backward.restype = i32
    dec = [vp, vp, vp, vp, _Strides, _Strides, vp, i32, i32, i32, i32, i32, i32, f32, f32]
    L.llla_decode.argtypes = dec + [vp, sz, vp]
    L.llla_decode.restype = i32
    L.llla_decode_path.argtypes = dec + [i32, vp, sz, vp]
    L.llla_decode_path.restype = i32
    L.llla_decode_static.argtypes = dec + [vp]
    L.llla_decode_static.restype = i32
    L.llla_status_string.argtypes = [i32]
    L.llla_status_string.restype = ctypes.c_char_p
    L.llla_version.restype = ctypes.c_char_p
    if measure:
        L.llla_profile_enable.argtypes = [i32]
        L.llla_profile_enable.restype = None
        L.llla_profile_last.argtypes = [ctypes.POINTER(f32), ctypes.POINTER(ctypes.c_char_p), i32]
        L.llla_profile_last.restype = i32
        L.llla_probe_mfma_f16.argtypes = [i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.llla_probe_mfma_f16.restype = i32
        L.llla_probe_copy.argtypes = [vp, vp, sz, vp]
        L.llla_probe_copy.restype = i32


def _load(measure: bool):
    """Loads a built library.  A library that is missing, or whose stamp says it was built from other sources than
    the ones in the tree now, is rebuilt first (hipcc cross-compiles without a GPU); without a compiler that is an
    error -- a stale library is never loaded silently."""
    if measure in _libs:
        return _libs[measure]
    from . import build as _build
    path = _MEASURE_PATH if measure else _LIB_PATH
    if not _build.is_current(path, measure):
        if not os.path.exists(_build.HIPCC):
            raise RuntimeError("%s is missing or older than its sources and there is no hipcc to rebuild it" % path)
        _build._build_one(path, measure, False, ())
    L = ctypes.CDLL(path)
    _declare(L, measure)
    _libs[measure] = L
    return L


def lib():
    """The loaded C-ABI library (the production one unless use_measure_library(True) is in effect)."""
    return _load(_use_measure)


def measure_lib():
    return _load(True)


def status_string(code: int) -> str:
    return lib().llla_status_string(int(code)).decode()


def version() -> str:
    return lib().llla_version().decode()


def profile_enable(on: bool) -> None:
    """Measurement library only: record HIP events around every kernel of the following calls."""
    measure_lib().llla_profile_enable(1 if on else 0)


def profile_last() -> dict:
    """Measurement library only: stage name -> milliseconds of the most recent profiled call (waits for it)."""
    ms = (ctypes.c_float * 16)()
    names = (ctypes.c_char_p * 16)()
    k = measure_lib().llla_profile_last(ms, names, 16)
    return {names[i].decode(): float(ms[i]) for i in range(k)}


def probe_mfma_f16(iters: int, scratch) -> float:
    """Measurement library only: enqueue the pure-MFMA probe on the current stream; returns its flop count."""
    flops = ctypes.c_double(0.0)
    st = measure_lib().llla_probe_mfma_f16(int(iters), ctypes.c_void_p(scratch.data_ptr()), ctypes.byref(flops),
                                           ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if st != 0:
        raise LlaError(st, status_string(st))
    return float(flops.value)


def probe_copy(src, dst) -> int:
    """Measurement library only: enqueue one plain copy src -> dst (contiguous device tensors of equal byte size) on
    the current stream; returns the bytes copied (that many read, that many written)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("probe_copy needs two contiguous tensors of the same size in bytes")
    st = measure_lib().llla_probe_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), ctypes.c_size_t(nbytes),
                                       ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if st != 0:
        raise LlaError(st, status_string(st))
    return nbytes


def forward_workspace_bytes(B, H, n, d, dtype) -> int:
    return int(lib().llla_forward_workspace_bytes(B, H, n, d, _DTYPES[dtype]))


def decode_workspace_bytes(B, H, L_max, d, dtype) -> int:
    return int(lib().llla_decode_workspace_bytes(B, H, L_max, d, _DTYPES[dtype]))


def _strides4(t: torch.Tensor) -> _Strides:
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("expected a [B, H, n, d] tensor with unit stride along d")
    return _Strides(t.stride(0), t.stride(1), t.stride(2))


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _workspace(nbytes: int, device, workspace):
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    return workspace


def _on_callers_stream(fn):
    """Runs `fn` with its ``stream`` argument as torch's current stream.  The scratch and output tensors it allocates
    then belong to that stream: torch's caching allocator hands a freed block only to later work of the stream it was
    allocated on, so the scratch is not reused while the library's kernels, enqueued on that same stream, still
    touch it."""
    @functools.wraps(fn)
    def wrapped(*args, **kw):
        stream = kw.get("stream")
        if stream is None:
            return fn(*args, **kw)
        with torch.cuda.stream(stream):
            return fn(*args, **kw)
    return wrapped


@_on_callers_stream
def llla_forward(Q, K, V, lam, scale: float, causal: bool = True, out_dtype=None, path: str = "auto",
                 workspace=None, out=None, stream=None, return_stats: bool = False):
    """O = LLA(Q, K, V) for [B, H, n, d] device tensors (f32 or bf16).  ``lam`` is a float or a device float32
    tensor [B, H, n] (one ridge per query row).  Returns O ([B, H, n, d]), or (O, rho, delta) with the per-row
    statistics of Eq. (lla) when ``return_stats`` is set."""
    if not (Q.is_cuda and K.is_cuda and V.is_cuda):
        raise ValueError("llla_forward needs device tensors; this library has no CPU path")
    if not (Q.dtype == K.dtype == V.dtype) or Q.dtype not in _DTYPES:
        raise ValueError("Q, K, V must share dtype float32 or bfloat16")
    B, H, n, d = Q.shape
    if K.shape != Q.shape or V.shape != Q.shape:
        raise ValueError("Q, K, V must have the same [B, H, n, d] shape")
    lam_rows = None
    if torch.is_tensor(lam):
        lam_rows = lam
        if not (lam_rows.is_cuda and lam_rows.dtype == torch.float32 and tuple(lam_rows.shape) == (B, H, n)
                and lam_rows.is_contiguous()):
            raise ValueError("a per-row ridge must be a contiguous device float32 tensor [B, H, n]")
    out_dtype = torch.float32 if out_dtype is None else out_dtype
    O = torch.empty((B, H, n, d), dtype=out_dtype, device=Q.device) if out is None else out
    rho = torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device) if return_stats else None
    delta = torch.empty((B, H, n), dtype=torch.float32, device=Q.device) if return_stats else None
    L = lib()
    need = forward_workspace_bytes(B, H, n, d, Q.dtype)
    ws = _workspace(need, Q.device, workspace)
    st = L.llla_forward_ex(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                           _strides4(Q), _strides4(K), _strides4(V), _strides4(O),
                           B, H, n, d, _DTYPES[Q.dtype], _DTYPES[O.dtype], 1 if causal else 0,
                           0.0 if lam_rows is not None else float(lam),
                           None if lam_rows is None else lam_rows.data_ptr(), float(scale),
                           None if rho is None else rho.data_ptr(), None if delta is None else delta.data_ptr(),
                           PATHS[path], ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream))
    if st != 0:
        raise LlaError(st, "llla_forward")
    return (O, rho, delta) if return_stats else O


def forward_cg_workspace_bytes(B, H, n, d, dtype) -> int:
    return int(lib().llla_forward_cg_workspace_bytes(B, H, n, d, _DTYPES[dtype]))


@_on_callers_stream
def llla_forward_cg(Q, K, V, lam: float, scale: float, max_steps: int, eps: float = 0.0, out_dtype=None,
                    workspace=None, out=None, stream=None, return_stats: bool = False):
    """The paper's approximate forward: rho from at most ``max_steps`` conjugate-gradient steps (bf16,
    causal).  Returns O, or (O, rho, delta, steps) with ``return_stats``."""
    if not (Q.is_cuda and K.is_cuda and V.is_cuda):
        raise ValueError("llla_forward_cg needs device tensors; this library has no CPU path")
    if not (Q.dtype == K.dtype == V.dtype) or Q.dtype not in _DTYPES:
        raise ValueError("Q, K, V must share dtype float32 or bfloat16")
    B, H, n, d = Q.shape
    if K.shape != Q.shape or V.shape != Q.shape:
        raise ValueError("Q, K, V must have the same [B, H, n, d] shape")
    out_dtype = torch.float32 if out_dtype is None else out_dtype
    O = torch.empty((B, H, n, d), dtype=out_dtype, device=Q.device) if out is None else out
    rho = torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device) if return_stats else None
    delta = torch.empty((B, H, n), dtype=torch.float32, device=Q.device) if return_stats else None
    steps = torch.empty((B, H, n), dtype=torch.int32, device=Q.device) if return_stats else None
    need = forward_cg_workspace_bytes(B, H, n, d, Q.dtype)
    ws = _workspace(need, Q.device, workspace)
    st = lib().llla_forward_cg(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                               _strides4(Q), _strides4(K), _strides4(V), _strides4(O),
                               B, H, n, d, _DTYPES[Q.dtype], _DTYPES[O.dtype], float(lam), float(scale),
                               int(max_steps), float(eps),
                               None if rho is None else rho.data_ptr(), None if delta is None else delta.data_ptr(),
                               None if steps is None else steps.data_ptr(),
                               ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream))
    if st != 0:
        raise LlaError(st, "llla_forward_cg")
    return (O, rho, delta, steps) if return_stats else O


def backward_workspace_bytes(B, H, n, d, dtype) -> int:
    return int(lib().llla_backward_workspace_bytes(B, H, n, d, _DTYPES[dtype]))


@_on_callers_stream
def llla_backward(Q, K, V, dO, lam, scale: float, path: str = "auto", workspace=None, stream=None,
                  return_dlambda: bool = False, out=None):
    """Gradients of sum(dO * llla_forward(Q, K, V)) (causal): returns (dQ, dK, dV) as float32 [B, H, n, d], plus
    dL/dlambda per row [B, H, n] with ``return_dlambda``.  ``lam`` as in ``llla_forward``; dO has the dtype of Q.
    ``out``: optional (dQ, dK, dV) or (dQ, dK, dV, dlambda) tensors to write into."""
    if not (Q.is_cuda and K.is_cuda and V.is_cuda and dO.is_cuda):
        raise ValueError("llla_backward needs device tensors; this library has no CPU path")
    if not (Q.dtype == K.dtype == V.dtype == dO.dtype) or Q.dtype not in _DTYPES:
        raise ValueError("Q, K, V, dO must share dtype float32 or bfloat16")
    B, H, n, d = Q.shape
    if K.shape != Q.shape or V.shape != Q.shape or dO.shape != Q.shape:
        raise ValueError("Q, K, V, dO must have the same [B, H, n, d] shape")
    lam_rows = None
    if torch.is_tensor(lam):
        lam_rows = lam
        if not (lam_rows.is_cuda and lam_rows.dtype == torch.float32 and tuple(lam_rows.shape) == (B, H, n)
                and lam_rows.is_contiguous()):
            raise ValueError("a per-row ridge must be a contiguous device float32 tensor [B, H, n]")
    if out is not None:
        dQ, dK, dV = out[:3]
        dlam = out[3] if len(out) > 3 else None
        for t in (dQ, dK, dV):
            if not (t.is_cuda and t.dtype == torch.float32 and tuple(t.shape) == (B, H, n, d) and t.is_contiguous()):
                raise ValueError("gradient outputs must be contiguous device float32 tensors [B, H, n, d]")
        if dlam is not None and not (dlam.is_cuda and dlam.dtype == torch.float32 and tuple(dlam.shape) == (B, H, n)
                                     and dlam.is_contiguous()):
            raise ValueError("dlambda must be a contiguous device float32 tensor [B, H, n]")
        return_dlambda = dlam is not None
    else:
        dQ, dK, dV = (torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device) for _ in range(3))
        dlam = torch.empty((B, H, n), dtype=torch.float32, device=Q.device) if return_dlambda else None
    need = backward_workspace_bytes(B, H, n, d, Q.dtype)
    ws = _workspace(need, Q.device, workspace)
    st = lib().llla_backward(Q.data_ptr(), K.data_ptr(), V.data_ptr(), dO.data_ptr(),
                             _strides4(Q), _strides4(K), _strides4(V), _strides4(dO),
                             dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), None if dlam is None else dlam.data_ptr(),
                             B, H, n, d, _DTYPES[Q.dtype], 0.0 if lam_rows is not None else float(lam),
                             None if lam_rows is None else lam_rows.data_ptr(), float(scale), PATHS[path],
                             ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream))
    if st != 0:
        raise LlaError(st, "llla_backward")
    return (dQ, dK, dV, dlam) if return_dlambda else (dQ, dK, dV)


@_on_callers_stream
def llla_decode(q, Kc, Vc, lam: float, scale: float, seqlens=None, out_dtype=None, path: str = "auto",
                workspace=None, out=None, stream=None):
    """One query per (batch, head) against [B, H, L_max, d] caches.  q: [B, H, d].  Returns [B, H, d]."""
    if not (q.is_cuda and Kc.is_cuda and Vc.is_cuda):
        raise ValueError("llla_decode needs device tensors; this library has no CPU path")
    if not (q.dtype == Kc.dtype == Vc.dtype) or q.dtype not in _DTYPES:
        raise ValueError("q, Kc, Vc must share dtype float32 or bfloat16")
    B, H, Lmax, d = Kc.shape
    if tuple(q.shape) != (B, H, d) or Vc.shape != Kc.shape or not q.is_contiguous():
        raise ValueError("q must be contiguous [B, H, d]; caches [B, H, L_max, d]")
    if seqlens is not None and (seqlens.dtype != torch.int32 or not seqlens.is_cuda or seqlens.numel() != B):
        raise ValueError("seqlens must be a device int32 tensor of B entries")
    out_dtype = torch.float32 if out_dtype is None else out_dtype
    o = torch.empty((B, H, d), dtype=out_dtype, device=q.device) if out is None else out
    L = lib()
    need = decode_workspace_bytes(B, H, Lmax, d, q.dtype)
    ws = _workspace(need, q.device, workspace)
    st = L.llla_decode_path(q.data_ptr(), Kc.data_ptr(), Vc.data_ptr(), o.data_ptr(),
                            _strides4(Kc), _strides4(Vc),
                            0 if seqlens is None else seqlens.data_ptr(),
                            B, H, Lmax, d, _DTYPES[q.dtype], _DTYPES[o.dtype],
                            float(lam), float(scale), PATHS[path],
                            ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream))
    if st != 0:
        raise LlaError(st, "llla_decode")
    return o


def llla_decode_static(q, Kc, Vc, lam: float, scale: float, out, seqlens=None, stream=None):
    """llla_decode without a workspace (the library's own fixed device array holds the partial records): for callers
    that may not allocate.  Nothing is allocated here either: ``out`` ([B, H, d], float32 or bfloat16) is required."""
    if not (q.is_cuda and Kc.is_cuda and Vc.is_cuda and out.is_cuda):
        raise ValueError("llla_decode_static needs device tensors; this library has no CPU path")
    if not (q.dtype == Kc.dtype == Vc.dtype) or q.dtype not in _DTYPES or out.dtype not in _DTYPES:
        raise ValueError("q, Kc, Vc must share dtype float32 or bfloat16")
    B, H, Lmax, d = Kc.shape
    if tuple(q.shape) != (B, H, d) or Vc.shape != Kc.shape or not q.is_contiguous():
        raise ValueError("q must be contiguous [B, H, d]; caches [B, H, L_max, d]")
    if tuple(out.shape) != (B, H, d) or not out.is_contiguous():
        raise ValueError("out must be contiguous [B, H, d]")
    if seqlens is not None and (seqlens.dtype != torch.int32 or not seqlens.is_cuda or seqlens.numel() != B):
        raise ValueError("seqlens must be a device int32 tensor of B entries")
    st = lib().llla_decode_static(q.data_ptr(), Kc.data_ptr(), Vc.data_ptr(), out.data_ptr(),
                                  _strides4(Kc), _strides4(Vc), 0 if seqlens is None else seqlens.data_ptr(),
                                  B, H, Lmax, d, _DTYPES[q.dtype], _DTYPES[out.dtype], float(lam), float(scale),
                                  _stream_ptr(stream))
    if st != 0:
        raise LlaError(st, "llla_decode_static")
    return out
