"""ctypes binding of libltn_attn.so: argument marshalling only.

Every function has the name and meaning of the C entry point in include/ltn_attn.h.
PyTorch is used for device memory and the current HIP stream; all arithmetic of the
attention path runs inside the library's kernels.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libltn_attn.so")
_lib = None

LTN_F32, LTN_BF16 = 0, 1
SYMBOLS = (
    "ltn_attn_fwd", "ltn_attn_fwd_gated", "ltn_attn_fwd_tiled", "ltn_gate_fwd", "ltn_gate_bwd",
    "ltn_attn_bwd", "ltn_attn_decode_step", "ltn_attn_decode_steps", "ltn_attn_pick_block",
    "ltn_attn_workspace_bytes", "ltn_attn_check_decay", "ltn_status_str",
    "ltn_prologue_fwd", "ltn_prologue_bwd", "ltn_prologue_workspace_bytes",
    "ltn_attn_fwd_dkdv", "ltn_attn_bwd_dkdv", "ltn_attn_decode_steps_dkdv",
    "ltn_attn_query_plan", "ltn_attn_set_debug_plan", "ltn_attn_fwd_static", "ltn_attn_bwd_tiled", "ltn_probe_stream_read", "ltn_attn_workspace_bytes_dkdv",
)


class LtnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = int(code)
        super().__init__(f"{where}: {ltn_status_str(code)}")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Open the built library; build it first only if nothing is built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build_library
        build_library(force=True)
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with __graft_entry__.build()")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, fp, ci, cl, sz = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong, ctypes.c_size_t
    lib.ltn_attn_fwd.argtypes = [vp, vp, vp, vp, fp, fp, fp, ci, ci, cl, ci, ci, ci, vp, sz, vp]
    lib.ltn_attn_fwd.restype = ci
    cf = ctypes.c_float
    lib.ltn_attn_fwd_gated.argtypes = [vp, vp, vp, vp, vp, vp, fp, fp, fp, cf, ci, ci, cl, ci, ci, ci, vp, sz, vp]
    lib.ltn_attn_fwd_gated.restype = ci
    lib.ltn_attn_fwd_tiled.argtypes = [vp, vp, vp, vp, fp, ci, ci, cl, ci, ci, vp]
    lib.ltn_attn_fwd_tiled.restype = ci
    lib.ltn_attn_bwd_tiled.argtypes = [vp, vp, vp, vp, vp, vp, vp, fp, ci, ci, cl, ci, ci, vp]
    lib.ltn_attn_bwd_tiled.restype = ci
    lib.ltn_gate_fwd.argtypes = [vp, vp, vp, cf, cl, ci, ci, vp]
    lib.ltn_gate_fwd.restype = ci
    lib.ltn_gate_bwd.argtypes = [vp, vp, vp, vp, vp, cf, cl, ci, ci, vp]
    lib.ltn_gate_bwd.restype = ci
    lib.ltn_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, fp, ci, ci, cl, ci, ci, ci, vp, sz, vp]
    lib.ltn_attn_bwd.restype = ci
    lib.ltn_attn_decode_step.argtypes = [vp, vp, vp, vp, fp, fp, ci, ci, ci, ci, vp]
    lib.ltn_attn_decode_step.restype = ci
    lib.ltn_attn_decode_steps.argtypes = [vp, vp, vp, vp, fp, fp, ci, ci, ci, ci, ci, vp]
    lib.ltn_attn_decode_steps.restype = ci
    lib.ltn_attn_pick_block.argtypes = [ci, ci]
    lib.ltn_attn_pick_block.restype = ci
    lib.ltn_attn_workspace_bytes.argtypes = [ci, ci, cl, ci, ci, ci, ci]
    lib.ltn_attn_workspace_bytes.restype = sz
    lib.ltn_attn_check_decay.argtypes = [ctypes.POINTER(ctypes.c_float), ci]
    lib.ltn_attn_check_decay.restype = ci
    lib.ltn_status_str.argtypes = [ci]
    lib.ltn_status_str.restype = ctypes.c_char_p
    lib.ltn_prologue_fwd.argtypes = [vp, fp, vp, ci, ci, ci, cl, ci, cl, ci, vp]
    lib.ltn_prologue_fwd.restype = ci
    lib.ltn_prologue_bwd.argtypes = [vp, fp, vp, vp, fp, ci, ci, ci, cl, ci, cl, ci, vp, sz, vp]
    lib.ltn_prologue_bwd.restype = ci
    lib.ltn_prologue_workspace_bytes.argtypes = [ci, ci, cl, ci]
    lib.ltn_prologue_workspace_bytes.restype = sz
    lib.ltn_attn_fwd_dkdv.argtypes = [vp, vp, vp, vp, fp, fp, fp, ci, ci, cl, ci, ci, ci, ci, vp, sz, vp]
    lib.ltn_attn_fwd_dkdv.restype = ci
    lib.ltn_attn_bwd_dkdv.argtypes = [vp, vp, vp, vp, vp, vp, vp, fp, ci, ci, cl, ci, ci, ci, ci, vp, sz, vp]
    lib.ltn_attn_workspace_bytes_dkdv.argtypes = [ci, ci, cl, ci, ci, ci, ci]
    lib.ltn_attn_workspace_bytes_dkdv.restype = sz
    lib.ltn_attn_bwd_dkdv.restype = ci
    lib.ltn_attn_decode_steps_dkdv.argtypes = [vp, vp, vp, vp, fp, fp, ci, ci, ci, ci, ci, ci, vp]
    lib.ltn_attn_decode_steps_dkdv.restype = ci
    lib.ltn_attn_fwd_static.argtypes = [vp, vp, vp, vp, fp, fp, fp, ci, ci, cl, ci, ci, ci, vp]
    lib.ltn_attn_fwd_static.restype = ci
    lib.ltn_probe_stream_read.argtypes = [vp, sz, sz, ci, ci, ci, vp, vp]
    lib.ltn_probe_stream_read.restype = ci
    lib.ltn_attn_query_plan.argtypes = [ci, ci, cl, ci, ci, ci, ctypes.POINTER(ci), ctypes.POINTER(ci)]
    lib.ltn_attn_query_plan.restype = ci
    lib.ltn_attn_set_debug_plan.argtypes = [ci, ci]
    lib.ltn_attn_set_debug_plan.restype = ci
    _lib = lib
    return lib


def ltn_status_str(code: int) -> str:
    return load_library().ltn_status_str(int(code)).decode()


def ltn_attn_pick_block(D: int, dtype: torch.dtype) -> int:
    return int(load_library().ltn_attn_pick_block(int(D), _dtype_code(dtype)))


def ltn_attn_workspace_bytes(Bt, H, N, D, block, dtype, call) -> int:
    """call: 0 = ltn_attn_fwd, 1 = ltn_attn_bwd, 2 = ltn_attn_fwd_gated."""
    return int(load_library().ltn_attn_workspace_bytes(Bt, H, N, D, block, _dtype_code(dtype), int(call)))


def ltn_attn_query_plan(Bt, H, N, D, dtype, call):
    """(value columns per workgroup, segments per chain) the library takes for these arguments."""
    dv, segs = ctypes.c_int(0), ctypes.c_int(0)
    rc = load_library().ltn_attn_query_plan(int(Bt), int(H), int(N), int(D), _dtype_code(dtype), int(call),
                                            ctypes.byref(dv), ctypes.byref(segs))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_query_plan")
    return dv.value, segs.value


def ltn_attn_set_debug_plan(dv=0, segs=0) -> None:
    """Test only: force the value-column split and the segment count (0 = the library's choice)."""
    rc = load_library().ltn_attn_set_debug_plan(int(dv), int(segs))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_set_debug_plan")


def ltn_attn_workspace_bytes_dkdv(Bt, H, N, Dk, Dv, dtype, call) -> int:
    """call: 0 = ltn_attn_fwd_dkdv, 1 = ltn_attn_bwd_dkdv."""
    return int(load_library().ltn_attn_workspace_bytes_dkdv(Bt, H, N, Dk, Dv, _dtype_code(dtype), int(call)))


def ltn_attn_check_decay(decay) -> int:
    """Validate a decay array (copied to the host); returns the status code."""
    d = torch.as_tensor(decay).detach().to("cpu", torch.float32).contiguous()
    buf = (ctypes.c_float * d.numel())(*d.tolist())
    return int(load_library().ltn_attn_check_decay(buf, d.numel()))


def _dtype_code(dtype: torch.dtype) -> int:
    if dtype == torch.float32:
        return LTN_F32
    if dtype == torch.bfloat16:
        return LTN_BF16
    raise TypeError(f"unsupported dtype {dtype}: the library computes in fp32 or bf16")


def _dev(t: torch.Tensor, what: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{what} must live on the GPU (the library has no CPU path)")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(device) -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def _workspace(nbytes: int, device):
    return None if nbytes == 0 else torch.empty(nbytes, dtype=torch.uint8, device=device)


def ltn_attn_fwd(q, k, v, decay, kv_in=None, return_state=False, block=0, out=None, kv_out=None):
    """O[Bt,H,N,D] = ((Q K^T) (.) M) V, optionally continuing from / returning the fp32 state."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (decay, "decay")):
        _dev(t, n)
    if q.shape != k.shape or q.shape != v.shape or q.dim() != 4 or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must be [Bt,H,N,D] tensors of one shape and dtype")
    Bt, H, N, D = q.shape
    if decay.dtype != torch.float32 or decay.numel() != H:
        raise ValueError("decay must be fp32 [H]")
    o = torch.empty_like(q) if out is None else _dev(out, "out")
    if kv_in is not None:
        _dev(kv_in, "kv_in")
        if kv_in.dtype != torch.float32 or tuple(kv_in.shape) != (Bt, H, D, D):
            raise ValueError("kv_in must be fp32 [Bt,H,D,D]")
    if kv_out is None and return_state:
        kv_out = torch.empty((Bt, H, D, D), dtype=torch.float32, device=q.device)
    code = _dtype_code(q.dtype)
    ws_bytes = int(lib.ltn_attn_workspace_bytes(Bt, H, N, D, block, code, 0))
    ws = _workspace(ws_bytes, q.device)
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(decay), _ptr(kv_in), _ptr(kv_out),
                              Bt, H, N, D, int(block), code, _ptr(ws), ws_bytes, _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_fwd")
    return (o, kv_out) if (return_state or kv_out is not None) else o


def ltn_attn_fwd_static(q, k, v, decay, out, kv_in=None, kv_out=None, block=0):
    """ltn_attn_fwd through the library's static scratch: every buffer comes from the caller,
    nothing is allocated here or in the library.  Returns `out`."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (decay, "decay"), (out, "out")):
        _dev(t, n)
    if q.shape != k.shape or q.shape != v.shape or q.shape != out.shape or q.dim() != 4:
        raise ValueError("q, k, v, out must be [Bt,H,N,D] tensors of one shape")
    if not (q.dtype == k.dtype == v.dtype == out.dtype):
        raise ValueError("q, k, v, out must share a dtype")
    Bt, H, N, D = q.shape
    if decay.dtype != torch.float32 or decay.numel() != H:
        raise ValueError("decay must be fp32 [H]")
    for t, n in ((kv_in, "kv_in"), (kv_out, "kv_out")):
        if t is not None:
            _dev(t, n)
            if t.dtype != torch.float32 or tuple(t.shape) != (Bt, H, D, D):
                raise ValueError(f"{n} must be fp32 [Bt,H,D,D]")
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_fwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(decay), _ptr(kv_in), _ptr(kv_out),
                                     Bt, H, N, D, int(block), _dtype_code(q.dtype), _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_fwd_static")
    return out


def ltn_attn_fwd_gated(q, k, v, u, decay, eps=0.0, kv_in=None, return_state=False, store_o=True, block=0,
                       out=None, y_out=None, kv_out=None):
    """Forward with the fused epilogue y = SRMSNorm_D(o) (.) u.  Returns (o or None, y[, kv_out])."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (u, "u"), (decay, "decay")):
        _dev(t, n)
    if not (q.shape == k.shape == v.shape == u.shape) or q.dim() != 4:
        raise ValueError("q, k, v, u must be [Bt,H,N,D] tensors of one shape")
    if not (q.dtype == k.dtype == v.dtype == u.dtype):
        raise ValueError("q, k, v, u must share a dtype")
    Bt, H, N, D = q.shape
    if decay.dtype != torch.float32 or decay.numel() != H:
        raise ValueError("decay must be fp32 [H]")
    o = (torch.empty_like(q) if out is None else _dev(out, "out")) if store_o else None
    y = torch.empty_like(q) if y_out is None else _dev(y_out, "y_out")
    if kv_in is not None:
        _dev(kv_in, "kv_in")
        if kv_in.dtype != torch.float32 or tuple(kv_in.shape) != (Bt, H, D, D):
            raise ValueError("kv_in must be fp32 [Bt,H,D,D]")
    if kv_out is None and return_state:
        kv_out = torch.empty((Bt, H, D, D), dtype=torch.float32, device=q.device)
    code = _dtype_code(q.dtype)
    ws_bytes = int(lib.ltn_attn_workspace_bytes(Bt, H, N, D, block, code, 2))
    ws = _workspace(ws_bytes, q.device)
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_fwd_gated(_ptr(q), _ptr(k), _ptr(v), _ptr(u), _ptr(o), _ptr(y), _ptr(decay),
                                    _ptr(kv_in), _ptr(kv_out), float(eps), Bt, H, N, D, int(block), code,
                                    _ptr(ws), ws_bytes, _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_fwd_gated")
    return (o, y, kv_out) if (return_state or kv_out is not None) else (o, y)


def _rows(x, what):
    _dev(x, what)
    if x.dim() < 1:
        raise ValueError(f"{what} must have a feature axis")
    return x.numel() // x.shape[-1] if x.numel() else 0, x.shape[-1]


def ltn_gate_fwd(x, u, eps=0.0, out=None):
    """y = x / sqrt(mean(x^2) + eps) (.) u over the last axis."""
    lib = load_library()
    rows, D = _rows(x, "x")
    _dev(u, "u")
    if u.shape != x.shape or u.dtype != x.dtype:
        raise ValueError("x and u must share shape and dtype")
    y = torch.empty_like(x) if out is None else _dev(out, "out")
    with torch.cuda.device(x.device):
        rc = lib.ltn_gate_fwd(_ptr(x), _ptr(u), _ptr(y), float(eps), rows, D, _dtype_code(x.dtype), _stream(x.device))
    if rc != 0:
        raise LtnError(rc, "ltn_gate_fwd")
    return y


def ltn_gate_bwd(x, u, d_y, eps=0.0, out=None):
    """(d_x, d_u) of ltn_gate_fwd."""
    lib = load_library()
    rows, D = _rows(x, "x")
    for t, n in ((u, "u"), (d_y, "d_y")):
        _dev(t, n)
        if t.shape != x.shape or t.dtype != x.dtype:
            raise ValueError("x, u and d_y must share shape and dtype")
    if out is None:
        dx, du = torch.empty_like(x), torch.empty_like(x)
    else:
        dx, du = (_dev(t, "out") for t in out)
    with torch.cuda.device(x.device):
        rc = lib.ltn_gate_bwd(_ptr(x), _ptr(u), _ptr(d_y), _ptr(dx), _ptr(du), float(eps), rows, D,
                              _dtype_code(x.dtype), _stream(x.device))
    if rc != 0:
        raise LtnError(rc, "ltn_gate_bwd")
    return dx, du


def ltn_attn_bwd(q, k, v, d_o, decay, block=0, out=None):
    """(dQ, dK, dV) of the forward definition; needs q, k, v, dO only."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (d_o, "d_o"), (decay, "decay")):
        _dev(t, n)
    if not (q.shape == k.shape == v.shape == d_o.shape) or q.dim() != 4:
        raise ValueError("q, k, v, d_o must be [Bt,H,N,D] tensors of one shape")
    if not (q.dtype == k.dtype == v.dtype == d_o.dtype):
        raise ValueError("q, k, v, d_o must share a dtype")
    Bt, H, N, D = q.shape
    if decay.dtype != torch.float32 or decay.numel() != H:
        raise ValueError("decay must be fp32 [H]")
    if out is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    else:
        dq, dk, dv = (_dev(t, "out") for t in out)
    code = _dtype_code(q.dtype)
    ws_bytes = int(lib.ltn_attn_workspace_bytes(Bt, H, N, D, block, code, 1))
    ws = _workspace(ws_bytes, q.device)
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(decay),
                              Bt, H, N, D, int(block), code, _ptr(ws), ws_bytes, _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_bwd")
    return dq, dk, dv


def ltn_attn_decode_step(q, k, v, kv, decay, out=None):
    """kv <- lambda kv + k^T v (in place); returns o = q kv.  q, k, v: [Bt,H,D]; kv: fp32 [Bt,H,D,D]."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (kv, "kv"), (decay, "decay")):
        _dev(t, n)
    if not (q.shape == k.shape == v.shape) or q.dim() != 3 or not (q.dtype == k.dtype == v.dtype):
        raise ValueError("q, k, v must be [Bt,H,D] tensors of one shape and dtype")
    Bt, H, D = q.shape
    if kv.dtype != torch.float32 or tuple(kv.shape) != (Bt, H, D, D):
        raise ValueError("kv must be fp32 [Bt,H,D,D]")
    if decay.dtype != torch.float32 or decay.numel() != H:
        raise ValueError("decay must be fp32 [H]")
    o = torch.empty_like(q) if out is None else _dev(out, "out")
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_decode_step(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(kv), _ptr(decay),
                                      Bt, H, D, _dtype_code(q.dtype), _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_decode_step")
    return o


def ltn_attn_decode_steps(q, k, v, kv, decay, out=None):
    """S decode steps in one call: q, k, v: [Bt,H,S,D]; kv: fp32 [Bt,H,D,D] updated in place; returns o."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (kv, "kv"), (decay, "decay")):
        _dev(t, n)
    if not (q.shape == k.shape == v.shape) or q.dim() != 4 or not (q.dtype == k.dtype == v.dtype):
        raise ValueError("q, k, v must be [Bt,H,S,D] tensors of one shape and dtype")
    Bt, H, S, D = q.shape
    if kv.dtype != torch.float32 or tuple(kv.shape) != (Bt, H, D, D):
        raise ValueError("kv must be fp32 [Bt,H,D,D]")
    if decay.dtype != torch.float32 or decay.numel() != H:
        raise ValueError("decay must be fp32 [H]")
    o = torch.empty_like(q) if out is None else _dev(out, "out")
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_decode_steps(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(kv), _ptr(decay),
                                       Bt, H, S, D, _dtype_code(q.dtype), _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_decode_steps")
    return o


def ltn_attn_fwd_tiled(q, k, v, decay, out=None):
    """The forward output by the quadratic tile loop of App. B Algorithm 3 (comparison kernel, bf16)."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (decay, "decay")):
        _dev(t, n)
    if q.shape != k.shape or q.shape != v.shape or q.dim() != 4 or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must be [Bt,H,N,D] tensors of one shape and dtype")
    Bt, H, N, D = q.shape
    if decay.dtype != torch.float32 or decay.numel() != H:
        raise ValueError("decay must be fp32 [H]")
    o = torch.empty_like(q) if out is None else _dev(out, "out")
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_fwd_tiled(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(decay), Bt, H, N, D,
                                    _dtype_code(q.dtype), _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_fwd_tiled")
    return o


def ltn_attn_bwd_tiled(q, k, v, d_o, decay, out=None):
    """(dQ, dK, dV) by the quadratic tile loops of App. B Algorithm 4 (comparison kernel, bf16)."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (d_o, "d_o"), (decay, "decay")):
        _dev(t, n)
    if not (q.shape == k.shape == v.shape == d_o.shape) or q.dim() != 4:
        raise ValueError("q, k, v, d_o must be [Bt,H,N,D] tensors of one shape")
    if not (q.dtype == k.dtype == v.dtype == d_o.dtype):
        raise ValueError("q, k, v, d_o must share a dtype")
    Bt, H, N, D = q.shape
    if decay.dtype != torch.float32 or decay.numel() != H:
        raise ValueError("decay must be fp32 [H]")
    if out is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    else:
        dq, dk, dv = (_dev(t, "out") for t in out)
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_bwd_tiled(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(decay),
                                    Bt, H, N, D, _dtype_code(q.dtype), _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_bwd_tiled")
    return dq, dk, dv


def ltn_probe_stream_read(buf, bytes_per_workgroup, workgroups, iters, to_registers=False, sink=None):
    """Measurement aid: enqueue the streaming-read probe on `buf` (a uint8 CUDA tensor)."""
    lib = load_library()
    _dev(buf, "buf")
    if sink is None:
        sink = torch.zeros(1, dtype=torch.int32, device=buf.device)
    with torch.cuda.device(buf.device):
        rc = lib.ltn_probe_stream_read(_ptr(buf), buf.numel() * buf.element_size(), int(bytes_per_workgroup), int(workgroups),
                                       int(iters), int(bool(to_registers)), _ptr(sink), _stream(buf.device))
    if rc != 0:
        raise LtnError(rc, "ltn_probe_stream_read")
    return sink


def ltn_prologue_workspace_bytes(Bt, H, N, D) -> int:
    return int(load_library().ltn_prologue_workspace_bytes(int(Bt), int(H), int(N), int(D)))


def _check_theta(theta, H, D):
    if theta is None:
        return
    _dev(theta, "theta")
    if theta.dtype != torch.float32 or tuple(theta.shape) != (H, D):
        raise ValueError("theta must be fp32 [H,D]")


def ltn_prologue_fwd(x, theta=None, act=True, pos0=0, out=None):
    """y = [z cos(theta p) | z sin(theta p)] with z = swish(x) (act) or x, p = pos0 + token; theta None: y = z."""
    lib = load_library()
    _dev(x, "x")
    if x.dim() != 4:
        raise ValueError("x must be [Bt,H,N,D]")
    Bt, H, N, D = x.shape
    _check_theta(theta, H, D)
    W = D if theta is None else 2 * D
    y = torch.empty((Bt, H, N, W), dtype=x.dtype, device=x.device) if out is None else _dev(out, "out")
    if tuple(y.shape) != (Bt, H, N, W) or y.dtype != x.dtype:
        raise ValueError("out must be [Bt,H,N,2D] (or [Bt,H,N,D] without theta) in x's dtype")
    with torch.cuda.device(x.device):
        rc = lib.ltn_prologue_fwd(_ptr(x), _ptr(theta), _ptr(y), int(bool(act)), Bt, H, N, D, int(pos0),
                                  _dtype_code(x.dtype), _stream(x.device))
    if rc != 0:
        raise LtnError(rc, "ltn_prologue_fwd")
    return y


def ltn_prologue_bwd(x, d_y, theta=None, act=True, pos0=0, want_dtheta=True):
    """(d_x, d_theta) of ltn_prologue_fwd for one tensor; d_theta is None without theta or when not wanted."""
    lib = load_library()
    _dev(x, "x")
    _dev(d_y, "d_y")
    if x.dim() != 4:
        raise ValueError("x must be [Bt,H,N,D]")
    Bt, H, N, D = x.shape
    _check_theta(theta, H, D)
    W = D if theta is None else 2 * D
    if tuple(d_y.shape) != (Bt, H, N, W) or d_y.dtype != x.dtype:
        raise ValueError("d_y must be [Bt,H,N,2D] (or [Bt,H,N,D] without theta) in x's dtype")
    dx = torch.empty_like(x)
    dth = torch.empty((H, D), dtype=torch.float32, device=x.device) if (theta is not None and want_dtheta) else None
    ws_bytes = int(lib.ltn_prologue_workspace_bytes(Bt, H, N, D)) if dth is not None else 0
    ws = _workspace(ws_bytes, x.device)
    with torch.cuda.device(x.device):
        rc = lib.ltn_prologue_bwd(_ptr(x), _ptr(theta), _ptr(d_y), _ptr(dx), _ptr(dth), int(bool(act)),
                                  Bt, H, N, D, int(pos0), _dtype_code(x.dtype), _ptr(ws), ws_bytes, _stream(x.device))
    if rc != 0:
        raise LtnError(rc, "ltn_prologue_bwd")
    return dx, dth


def _check_dkdv(q, k, v, decay):
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (decay, "decay")):
        _dev(t, n)
    if q.dim() != 4 or q.shape != k.shape or v.dim() != 4 or v.shape[:3] != q.shape[:3]:
        raise ValueError("q, k must be [Bt,H,N,Dk] and v [Bt,H,N,Dv]")
    if not (q.dtype == k.dtype == v.dtype):
        raise ValueError("q, k, v must share a dtype")
    Bt, H, N, Dk = q.shape
    if decay.dtype != torch.float32 or decay.numel() != H:
        raise ValueError("decay must be fp32 [H]")
    return Bt, H, N, Dk, v.shape[3]


def ltn_attn_fwd_dkdv(q, k, v, decay, kv_in=None, return_state=False, block=0, out=None, kv_out=None):
    """The forward with q, k of width Dk and v, o of width Dv (state fp32 [Bt,H,Dk,Dv])."""
    lib = load_library()
    Bt, H, N, Dk, Dv = _check_dkdv(q, k, v, decay)
    o = torch.empty_like(v) if out is None else _dev(out, "out")
    if kv_in is not None:
        _dev(kv_in, "kv_in")
        if kv_in.dtype != torch.float32 or tuple(kv_in.shape) != (Bt, H, Dk, Dv):
            raise ValueError("kv_in must be fp32 [Bt,H,Dk,Dv]")
    if kv_out is None and return_state:
        kv_out = torch.empty((Bt, H, Dk, Dv), dtype=torch.float32, device=q.device)
    code = _dtype_code(q.dtype)
    ws_bytes = int(lib.ltn_attn_workspace_bytes_dkdv(Bt, H, N, Dk, Dv, code, 0))
    ws = _workspace(ws_bytes, q.device)
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_fwd_dkdv(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(decay), _ptr(kv_in), _ptr(kv_out),
                                   Bt, H, N, Dk, Dv, int(block), code, _ptr(ws), ws_bytes, _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_fwd_dkdv")
    return (o, kv_out) if (return_state or kv_out is not None) else o


def ltn_attn_bwd_dkdv(q, k, v, d_o, decay, block=0):
    """(dQ, dK, dV) for q, k of width Dk and v, d_o of width Dv."""
    lib = load_library()
    Bt, H, N, Dk, Dv = _check_dkdv(q, k, v, decay)
    _dev(d_o, "d_o")
    if d_o.shape != v.shape or d_o.dtype != v.dtype:
        raise ValueError("d_o must have v's shape and dtype")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    code = _dtype_code(q.dtype)
    ws_bytes = int(lib.ltn_attn_workspace_bytes_dkdv(Bt, H, N, Dk, Dv, code, 1))
    ws = _workspace(ws_bytes, q.device)
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_bwd_dkdv(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(decay),
                                   Bt, H, N, Dk, Dv, int(block), code, _ptr(ws), ws_bytes, _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_bwd_dkdv")
    return dq, dk, dv


def ltn_attn_decode_steps_dkdv(q, k, v, kv, decay, out=None):
    """S decode steps: q, k [Bt,H,S,Dk]; v [Bt,H,S,Dv]; kv fp32 [Bt,H,Dk,Dv] updated in place; returns o."""
    lib = load_library()
    Bt, H, S, Dk, Dv = _check_dkdv(q, k, v, decay)
    _dev(kv, "kv")
    if kv.dtype != torch.float32 or tuple(kv.shape) != (Bt, H, Dk, Dv):
        raise ValueError("kv must be fp32 [Bt,H,Dk,Dv]")
    o = torch.empty_like(v) if out is None else _dev(out, "out")
    with torch.cuda.device(q.device):
        rc = lib.ltn_attn_decode_steps_dkdv(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(kv), _ptr(decay),
                                            Bt, H, S, Dk, Dv, _dtype_code(q.dtype), _stream(q.device))
    if rc != 0:
        raise LtnError(rc, "ltn_attn_decode_steps_dkdv")
    return o
