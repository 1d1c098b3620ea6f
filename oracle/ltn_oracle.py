"""ctypes loader for the fp64 CPU oracle of Lightning Attention (arXiv 2307.14995).

TEST INFRASTRUCTURE ONLY: the test suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; the GPU library never does, and
this module never imports the GPU package.

Every function takes array-likes (numpy arrays, or torch CPU tensors of any
float dtype, bf16 included), widens them exactly to float64 and returns float64
numpy arrays.  Tensor layout is ``[Bt, H, N, D]``; ``decay`` is ``[H]``; states
are ``[Bt, H, D, D]`` with rows indexed by the key feature.

The formulas are in ``ltn_oracle.c``; each entry below names the passage of the
paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ltn_oracle.c")
_LIB = os.path.join(_HERE, "libltn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (seconds).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ci, cl = ctypes.c_int, ctypes.c_longlong
        lib.ltn_oracle_num_threads.restype = ci
        lib.ltn_oracle_set_num_threads.argtypes = [ci]
        lib.ltn_oracle_fwd_quadratic.argtypes = [dp, dp, dp, dp, ci, ci, cl, ci, dp]
        lib.ltn_oracle_fwd_recurrent.argtypes = [dp, dp, dp, dp, dp, ci, ci, cl, ci, dp, dp]
        lib.ltn_oracle_fwd_origin.argtypes = [dp, dp, dp, dp, ci, ci, cl, ci, dp, dp]
        lib.ltn_oracle_fwd_tiled.argtypes = [dp, dp, dp, dp, ci, ci, cl, ci, ci, ci, dp]
        lib.ltn_oracle_fwd_block.argtypes = [dp, dp, dp, dp, dp, ci, ci, cl, ci, ci, dp, dp]
        lib.ltn_oracle_bwd_quadratic.argtypes = [dp, dp, dp, dp, dp, ci, ci, cl, ci, dp, dp, dp]
        lib.ltn_oracle_bwd_recurrent.argtypes = [dp, dp, dp, dp, dp, ci, ci, cl, ci, dp, dp, dp]
        lib.ltn_oracle_bwd_block.argtypes = [dp, dp, dp, dp, dp, ci, ci, cl, ci, ci, dp, dp, dp]
        lib.ltn_oracle_decode_step.argtypes = [dp, dp, dp, dp, ci, ci, ci, dp, dp]
        cd = ctypes.c_double
        lib.ltn_oracle_gate_fwd.argtypes = [dp, dp, cd, cl, ci, dp]
        lib.ltn_oracle_gate_bwd.argtypes = [dp, dp, dp, cd, cl, ci, dp, dp]
        lib.ltn_oracle_fwd_recurrent_dkdv.argtypes = [dp, dp, dp, dp, dp, ci, ci, cl, ci, ci, dp, dp]
        lib.ltn_oracle_bwd_recurrent_dkdv.argtypes = [dp, dp, dp, dp, dp, ci, ci, cl, ci, ci, dp, dp, dp]
        lib.ltn_oracle_decode_step_dkdv.argtypes = [dp, dp, dp, dp, ci, ci, ci, ci, dp, dp]
        lib.ltn_oracle_lrpe_fwd_quadratic.argtypes = [dp, dp, dp, dp, dp, ci, ci, cl, ci, dp]
        lib.ltn_oracle_prologue_fwd.argtypes = [dp, dp, ci, ci, ci, cl, ci, cl, dp]
        lib.ltn_oracle_prologue_bwd.argtypes = [dp, dp, dp, ci, ci, ci, cl, ci, cl, dp, dp]
        for name in ("fwd_recurrent_dkdv", "bwd_recurrent_dkdv", "decode_step_dkdv", "lrpe_fwd_quadratic",
                     "prologue_fwd", "prologue_bwd"):
            getattr(lib, "ltn_oracle_" + name).restype = None
        for name in ("gate_fwd", "gate_bwd", "fwd_quadratic", "fwd_recurrent", "fwd_origin", "fwd_tiled", "fwd_block",
                     "bwd_quadratic", "bwd_recurrent", "bwd_block", "decode_step",
                     "set_num_threads"):
            getattr(lib, "ltn_oracle_" + name).restype = None
        _lib = lib
    return _lib


def _f64(x) -> np.ndarray:
    """Exact widening to a contiguous float64 numpy array."""
    if hasattr(x, "detach"):  # torch tensor (numpy cannot hold bf16)
        x = x.detach().cpu().double().numpy()
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _shape4(q, k, v):
    assert q.ndim == 4 and q.shape == k.shape == v.shape, "expect [Bt,H,N,D] tensors of one shape"
    return q.shape


def num_threads() -> int:
    return int(_load().ltn_oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().ltn_oracle_set_num_threads(int(n))


def fwd_quadratic(q, k, v, decay):
    """Sec. 3.2.1 definition O = (Q K^T (.) M) V, M[t,s] = lambda^(t-s), t >= s."""
    q, k, v, decay = _f64(q), _f64(k), _f64(v), _f64(decay)
    Bt, H, N, D = _shape4(q, k, v)
    assert decay.shape == (H,)
    o = np.empty_like(q)
    _load().ltn_oracle_fwd_quadratic(_p(q), _p(k), _p(v), _p(decay), Bt, H, N, D, _p(o))
    return o


def fwd_recurrent(q, k, v, decay, kv_in=None, return_state=False):
    """Sec. 3.3 Algorithm 2: kv = lambda kv + k^T v; o = q kv, token by token."""
    q, k, v, decay = _f64(q), _f64(k), _f64(v), _f64(decay)
    Bt, H, N, D = _shape4(q, k, v)
    assert decay.shape == (H,)
    kvi = None if kv_in is None else _f64(kv_in)
    if kvi is not None:
        assert kvi.shape == (Bt, H, D, D)
    o = np.empty_like(q)
    kvo = np.empty((Bt, H, D, D), dtype=np.float64)
    _load().ltn_oracle_fwd_recurrent(_p(q), _p(k), _p(v), _p(decay), _p(kvi), Bt, H, N, D,
                                     _p(o), _p(kvo))
    return (o, kvo) if return_state else o


def fwd_origin(q, k, v, decay):
    """Sec. 3.3 Algorithm 1 (the overflow-prone factorisation); returns (o, kv_N)."""
    q, k, v, decay = _f64(q), _f64(k), _f64(v), _f64(decay)
    Bt, H, N, D = _shape4(q, k, v)
    o = np.empty_like(q)
    kvo = np.empty((Bt, H, D, D), dtype=np.float64)
    with np.errstate(all="ignore"):
        _load().ltn_oracle_fwd_origin(_p(q), _p(k), _p(v), _p(decay), Bt, H, N, D, _p(o), _p(kvo))
    return o, kvo


def fwd_tiled(q, k, v, decay, Br, Bc):
    """App. B Algorithm 3: quadratic (i, j) tile loops with block sizes Br, Bc."""
    q, k, v, decay = _f64(q), _f64(k), _f64(v), _f64(decay)
    Bt, H, N, D = _shape4(q, k, v)
    o = np.empty_like(q)
    _load().ltn_oracle_fwd_tiled(_p(q), _p(k), _p(v), _p(decay), Bt, H, N, D, int(Br), int(Bc), _p(o))
    return o


def fwd_block(q, k, v, decay, block, kv_in=None, return_state=False):
    """Blockwise re-association: masked intra tile + decayed running-state term."""
    q, k, v, decay = _f64(q), _f64(k), _f64(v), _f64(decay)
    Bt, H, N, D = _shape4(q, k, v)
    kvi = None if kv_in is None else _f64(kv_in)
    o = np.empty_like(q)
    kvo = np.empty((Bt, H, D, D), dtype=np.float64)
    _load().ltn_oracle_fwd_block(_p(q), _p(k), _p(v), _p(decay), _p(kvi), Bt, H, N, D, int(block),
                                 _p(o), _p(kvo))
    return (o, kvo) if return_state else o


def _bwd(fn, q, k, v, d_o, decay, *extra):
    q, k, v, d_o, decay = _f64(q), _f64(k), _f64(v), _f64(d_o), _f64(decay)
    Bt, H, N, D = _shape4(q, k, v)
    assert d_o.shape == q.shape and decay.shape == (H,)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    fn(_p(q), _p(k), _p(v), _p(d_o), _p(decay), Bt, H, N, D, *extra, _p(dq), _p(dk), _p(dv))
    return dq, dk, dv


def bwd_quadratic(q, k, v, d_o, decay):
    """Derivative of the definition: dV = A^T dO, dA = (dO V^T)(.)M, dQ = dA K, dK = dA^T Q."""
    return _bwd(_load().ltn_oracle_bwd_quadratic, q, k, v, d_o, decay)


def bwd_recurrent(q, k, v, d_o, decay):
    """Prefix-state sweep for dQ, reverse suffix-state sweep for dK and dV."""
    return _bwd(_load().ltn_oracle_bwd_recurrent, q, k, v, d_o, decay)


def bwd_block(q, k, v, d_o, decay, block):
    """Blockwise backward (forward-order sweep for dQ, reverse-order sweep for dK, dV)."""
    return _bwd(_load().ltn_oracle_bwd_block, q, k, v, d_o, decay, int(block))


def decode_step(q, k, v, kv, decay):
    """One iteration of Algorithm 2 on a given state; returns (o, new_kv)."""
    q, k, v, decay = _f64(q), _f64(k), _f64(v), _f64(decay)
    kv = _f64(kv).copy()
    Bt, H, D = q.shape
    assert kv.shape == (Bt, H, D, D) and decay.shape == (H,)
    o = np.empty_like(q)
    _load().ltn_oracle_decode_step(_p(q), _p(k), _p(v), _p(decay), Bt, H, D, _p(kv), _p(o))
    return o, kv


def gate_fwd(x, u, eps=0.0):
    """Eq. 3 with the SimpleRMSNorm of Sec. 3.1.3 over the last axis:
    y = x / sqrt(mean(x^2) + eps) * u."""
    x, u = _f64(x), _f64(u)
    assert x.shape == u.shape
    y = np.empty_like(x)
    d = x.shape[-1]
    _load().ltn_oracle_gate_fwd(_p(x), _p(u), float(eps), x.size // d, d, _p(y))
    return y


def gate_bwd(x, u, dy, eps=0.0):
    """Derivative of gate_fwd: returns (dx, du)."""
    x, u, dy = _f64(x), _f64(u), _f64(dy)
    assert x.shape == u.shape == dy.shape
    dx, du = np.empty_like(x), np.empty_like(x)
    d = x.shape[-1]
    _load().ltn_oracle_gate_bwd(_p(x), _p(u), _p(dy), float(eps), x.size // d, d, _p(dx), _p(du))
    return dx, du


def fwd_gated(q, k, v, u, decay, eps=0.0, kv_in=None):
    """Token mixer of Eq. 3: the attention output of the definition (Sec. 3.2.1), normalised
    per head and gated.  Returns (o, y)."""
    o = fwd_recurrent(q, k, v, decay, kv_in=kv_in) if kv_in is not None else fwd_quadratic(q, k, v, decay)
    return o, gate_fwd(o, u, eps)


# ---------------------------------------------------------------------------
# Query/key width Dk different from the value width Dv (q, k: [Bt,H,N,Dk];
# v, o: [Bt,H,N,Dv]; states [Bt,H,Dk,Dv]), and the input side of the token mixer.
# ---------------------------------------------------------------------------

def _shape_dkdv(q, k, v):
    assert q.ndim == 4 and q.shape == k.shape and v.shape[:3] == q.shape[:3], "expect q,k [Bt,H,N,Dk], v [Bt,H,N,Dv]"
    Bt, H, N, Dk = q.shape
    return Bt, H, N, Dk, v.shape[3]


def _mask(lam, N):
    """M[t,s] = lam^(t-s) for t >= s else 0 (Eq. 1 without the phase); 0^0 = 1."""
    t = np.arange(N)
    d = t[:, None] - t[None, :]
    with np.errstate(divide="ignore", invalid="ignore"):
        m = np.where(d >= 0, np.power(float(lam), np.maximum(d, 0).astype(np.float64)), 0.0)
    return m


def fwd_quadratic_dkdv(q, k, v, decay):
    """The definition (Sec. 3.2.1), O = ((Q K^T) (.) M) V, chain by chain with numpy
    matrix products; any Dk, Dv."""
    q, k, v, decay = _f64(q), _f64(k), _f64(v), _f64(decay)
    Bt, H, N, Dk, Dv = _shape_dkdv(q, k, v)
    o = np.empty((Bt, H, N, Dv))
    for b in range(Bt):
        for h in range(H):
            o[b, h] = ((q[b, h] @ k[b, h].T) * _mask(decay[h], N)) @ v[b, h]
    return o


def bwd_quadratic_dkdv(q, k, v, d_o, decay):
    """Derivative of the definition: with A = (Q K^T)(.)M and dA = (dO V^T)(.)M,
    dQ = dA K, dK = dA^T Q, dV = A^T dO; any Dk, Dv."""
    q, k, v, d_o, decay = _f64(q), _f64(k), _f64(v), _f64(d_o), _f64(decay)
    Bt, H, N, Dk, Dv = _shape_dkdv(q, k, v)
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    for b in range(Bt):
        for h in range(H):
            M = _mask(decay[h], N)
            A = (q[b, h] @ k[b, h].T) * M
            dA = (d_o[b, h] @ v[b, h].T) * M
            dq[b, h] = dA @ k[b, h]
            dk[b, h] = dA.T @ q[b, h]
            dv[b, h] = A.T @ d_o[b, h]
    return dq, dk, dv


def fwd_recurrent_dkdv(q, k, v, decay, kv_in=None, return_state=False):
    """Algorithm 2 (Sec. 3.3) with a [Dk x Dv] state."""
    q, k, v, decay = _f64(q), _f64(k), _f64(v), _f64(decay)
    Bt, H, N, Dk, Dv = _shape_dkdv(q, k, v)
    kv_in = None if kv_in is None else _f64(kv_in)
    assert kv_in is None or kv_in.shape == (Bt, H, Dk, Dv)
    o = np.empty((Bt, H, N, Dv))
    kv_out = np.empty((Bt, H, Dk, Dv)) if return_state else None
    _load().ltn_oracle_fwd_recurrent_dkdv(_p(q), _p(k), _p(v), _p(decay), _p(kv_in), Bt, H, N, Dk, Dv,
                                          _p(o), _p(kv_out))
    return (o, kv_out) if return_state else o


def bwd_recurrent_dkdv(q, k, v, d_o, decay):
    """Gradients by the two recurrent sweeps; returns (dq, dk, dv)."""
    q, k, v, d_o, decay = _f64(q), _f64(k), _f64(v), _f64(d_o), _f64(decay)
    Bt, H, N, Dk, Dv = _shape_dkdv(q, k, v)
    assert d_o.shape == v.shape
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    _load().ltn_oracle_bwd_recurrent_dkdv(_p(q), _p(k), _p(v), _p(d_o), _p(decay), Bt, H, N, Dk, Dv,
                                          _p(dq), _p(dk), _p(dv))
    return dq, dk, dv


def decode_step_dkdv(q, k, v, kv, decay):
    """One iteration of Algorithm 2 on a [Bt,H,Dk,Dv] state; returns (o, new_kv)."""
    q, k, v, decay = _f64(q), _f64(k), _f64(v), _f64(decay)
    kv = _f64(kv).copy()
    Bt, H, Dk = q.shape
    Dv = v.shape[2]
    assert kv.shape == (Bt, H, Dk, Dv) and decay.shape == (H,)
    o = np.empty_like(v)
    _load().ltn_oracle_decode_step_dkdv(_p(q), _p(k), _p(v), _p(decay), Bt, H, Dk, Dv, _p(kv), _p(o))
    return o, kv


def lrpe_fwd_quadratic(q, k, v, decay, theta):
    """Eq. 1 (LRPE-d) taken literally as the score, real part, feature-wise phase:
    a[t,s] = lam^(t-s) sum_d q_t[d] k_s[d] cos(theta[h,d] (t-s));  O = A V."""
    q, k, v, decay, theta = _f64(q), _f64(k), _f64(v), _f64(decay), _f64(theta)
    Bt, H, N, D = _shape4(q, k, v)
    assert theta.shape == (H, D)
    o = np.empty_like(q)
    _load().ltn_oracle_lrpe_fwd_quadratic(_p(q), _p(k), _p(v), _p(decay), _p(theta), Bt, H, N, D, _p(o))
    return o


def prologue_fwd(x, theta=None, act=True, pos0=0):
    """Input side of the token mixer for queries and keys: z = swish(x) (Eq. 2) when
    ``act``, then the separable form of Eq. 1's phase, y = [z cos(theta p) | z sin(theta p)]
    at absolute positions p = pos0 + token index (width 2D); theta None: y = z."""
    x = _f64(x)
    Bt, H, N, D = x.shape
    theta = None if theta is None else _f64(theta)
    assert theta is None or theta.shape == (H, D)
    y = np.empty((Bt, H, N, D if theta is None else 2 * D))
    _load().ltn_oracle_prologue_fwd(_p(x), _p(theta), int(bool(act)), Bt, H, N, D, int(pos0), _p(y))
    return y


def prologue_bwd(x, dy, theta=None, act=True, pos0=0):
    """Derivative of prologue_fwd: returns (dx, dtheta); dtheta is None without theta."""
    x, dy = _f64(x), _f64(dy)
    Bt, H, N, D = x.shape
    theta = None if theta is None else _f64(theta)
    assert dy.shape == (Bt, H, N, D if theta is None else 2 * D)
    dx = np.empty_like(x)
    dth = None if theta is None else np.empty((H, D))
    _load().ltn_oracle_prologue_bwd(_p(x), _p(theta), _p(dy), int(bool(act)), Bt, H, N, D, int(pos0),
                                    _p(dx), _p(dth))
    return dx, dth


def rel_l2(x, ref) -> float:
    """||x - ref||_2 / ||ref||_2 in fp64 over the whole tensor (0 if both are zero)."""
    x, ref = _f64(x), _f64(ref)
    den = float(np.linalg.norm(ref.ravel()))
    num = float(np.linalg.norm((x - ref).ravel()))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den


def max_rel_l2(x, ref) -> float:
    """Maximum of rel_l2 over the whole tensor and over every (b, h) slice."""
    x, ref = _f64(x), _f64(ref)
    worst = rel_l2(x, ref)
    if x.ndim >= 3:
        for b in range(x.shape[0]):
            for h in range(x.shape[1]):
                worst = max(worst, rel_l2(x[b, h], ref[b, h]))
    return worst
