"""Pins for the fp64 CPU oracle: every oracle function is checked against something
other than itself -- brute force written here in numpy, closed forms, textbook
special cases (cumulative sum, diagonal attention), the Algorithm 1 == Algorithm 2
identity proved in App. C, finite differences, and a hand-computed example.

Runs without a GPU.
"""
import os

import numpy as np
import pytest

from oracle import ltn_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def brute_force_fwd(q, k, v, decay):
    """O[t] = sum_{s<=t} lambda^(t-s) (q_t.k_s) v_s, pure Python loops (Sec. 3.2.1 + Eq. 1)."""
    Bt, H, N, D = q.shape
    o = np.zeros_like(q)
    for b in range(Bt):
        for h in range(H):
            lam = float(decay[h])
            for t in range(N):
                for s in range(t + 1):
                    w = 1.0
                    for _ in range(t - s):       # repeated multiplication: no pow, 0^0 = 1
                        w *= lam
                    dot = 0.0
                    for i in range(D):
                        dot += q[b, h, t, i] * k[b, h, s, i]
                    for j in range(D):
                        o[b, h, t, j] += w * dot * v[b, h, s, j]
    return o


def dense_mask(lam, N):
    t = np.arange(N)[:, None]
    s = np.arange(N)[None, :]
    with np.errstate(divide="ignore", invalid="ignore"):
        m = np.where(t >= s, np.power(float(lam), np.maximum(t - s, 0).astype(np.float64)), 0.0)
    m[np.arange(N), np.arange(N)] = 1.0
    return m


# --------------------------------------------------------------------------- forward


@pytest.mark.parametrize("N,D", [(1, 1), (1, 4), (2, 3), (7, 5), (16, 8)])
def test_fwd_quadratic_vs_brute_force(N, D):
    Bt, H = 2, 3
    q, k, v = rnd((Bt, H, N, D), 1), rnd((Bt, H, N, D), 2), rnd((Bt, H, N, D), 3)
    decay = np.array([0.9, 0.3, 1.0])
    ref = brute_force_fwd(q, k, v, decay)
    np.testing.assert_allclose(orc.fwd_quadratic(q, k, v, decay), ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(orc.fwd_recurrent(q, k, v, decay), ref, rtol=1e-11, atol=1e-12)


def test_hand_example_golden():
    """Three tokens, D = 1, lambda = 1/2, worked by hand from the definition."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "hand_example_n3_d1.txt"))
            if l.strip() and not l.startswith("#")]
    lam = float(rows[0][1])
    q = np.array([float(x) for x in rows[1][1:]]).reshape(1, 1, 3, 1)
    k = np.array([float(x) for x in rows[2][1:]]).reshape(1, 1, 3, 1)
    v = np.array([float(x) for x in rows[3][1:]]).reshape(1, 1, 3, 1)
    o = np.array([float(x) for x in rows[4][1:]]).reshape(1, 1, 3, 1)
    dq = np.array([float(x) for x in rows[5][1:]]).reshape(1, 1, 3, 1)
    dk = np.array([float(x) for x in rows[6][1:]]).reshape(1, 1, 3, 1)
    dv = np.array([float(x) for x in rows[7][1:]]).reshape(1, 1, 3, 1)
    decay = np.array([lam])
    for f in (orc.fwd_quadratic, orc.fwd_recurrent):
        np.testing.assert_allclose(f(q, k, v, decay), o, rtol=0, atol=1e-14)
    np.testing.assert_allclose(orc.fwd_block(q, k, v, decay, 2), o, rtol=0, atol=1e-14)
    np.testing.assert_allclose(orc.fwd_tiled(q, k, v, decay, 2, 1), o, rtol=0, atol=1e-14)
    ones = np.ones_like(q)   # dO = 1 everywhere
    for f in (orc.bwd_quadratic, orc.bwd_recurrent):
        g = f(q, k, v, ones, decay)
        np.testing.assert_allclose(g[0], dq, atol=1e-14)
        np.testing.assert_allclose(g[1], dk, atol=1e-14)
        np.testing.assert_allclose(g[2], dv, atol=1e-14)
    g = orc.bwd_block(q, k, v, ones, decay, 2)
    for a, b in zip(g, (dq, dk, dv)):
        np.testing.assert_allclose(a, b, atol=1e-14)


@pytest.mark.parametrize("lam", [0.0, 0.25, 0.9, 1.0])
def test_closed_form_all_ones(lam):
    """Q = K = V = 1  =>  O[t,j] = D * sum_{m=0..t} lambda^m (geometric series)."""
    N, D = 40, 6
    one = np.ones((1, 1, N, D))
    t = np.arange(N, dtype=np.float64)
    if lam == 1.0:
        expect = D * (t + 1)
    else:
        expect = D * (1 - lam ** (t + 1)) / (1 - lam)
    for f in (orc.fwd_quadratic, orc.fwd_recurrent):
        o = f(one, one, one, np.array([lam]))
        np.testing.assert_allclose(o[0, 0], np.repeat(expect[:, None], D, 1), rtol=1e-13)


def test_recurrent_equals_quadratic_long():
    Bt, H, N, D = 1, 4, 2048, 16
    q, k, v = (rnd((Bt, H, N, D), s) / 4 for s in (11, 12, 13))
    decay = np.array([0.43, 0.9, 0.9961, 1.0])
    a = orc.fwd_quadratic(q, k, v, decay)
    b = orc.fwd_recurrent(q, k, v, decay)
    assert orc.max_rel_l2(b, a) < 1e-12


def test_lambda_one_is_causal_cumsum():
    """lambda = 1 (the last layer's setting, Sec. 3.1.1): O_t = q_t . cumsum_s(k_s^T v_s)."""
    Bt, H, N, D = 1, 2, 33, 5
    q, k, v = rnd((Bt, H, N, D), 4), rnd((Bt, H, N, D), 5), rnd((Bt, H, N, D), 6)
    outer = np.einsum("bhni,bhnj->bhnij", k, v)
    state = np.cumsum(outer, axis=2)
    expect = np.einsum("bhni,bhnij->bhnj", q, state)
    decay = np.ones(H)
    np.testing.assert_allclose(orc.fwd_quadratic(q, k, v, decay), expect, rtol=1e-12, atol=1e-12)
    o, kv = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    np.testing.assert_allclose(o, expect, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(kv, state[:, :, -1], rtol=1e-12, atol=1e-12)


def test_lambda_zero_is_diagonal():
    """lambda = 0: only s = t survives, O_t = (q_t . k_t) v_t; lambda -> 0+ agrees."""
    Bt, H, N, D = 1, 2, 20, 7
    q, k, v = rnd((Bt, H, N, D), 7), rnd((Bt, H, N, D), 8), rnd((Bt, H, N, D), 9)
    expect = np.sum(q * k, axis=-1, keepdims=True) * v
    for lam in (0.0, 1e-30):
        decay = np.full(H, lam)
        for f in (orc.fwd_quadratic, orc.fwd_recurrent):
            np.testing.assert_allclose(f(q, k, v, decay), expect, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(orc.fwd_block(q, k, v, decay, 8), expect, rtol=1e-12, atol=1e-13)


def test_matrix_form_with_numpy_matmul():
    """(Q K^T (.) M) V with M built densely and the products done by numpy matmul."""
    Bt, H, N, D = 2, 2, 50, 9
    q, k, v = rnd((Bt, H, N, D), 21), rnd((Bt, H, N, D), 22), rnd((Bt, H, N, D), 23)
    decay = np.array([0.8, 0.05])
    expect = np.empty_like(q)
    for h in range(H):
        M = dense_mask(decay[h], N)
        expect[:, h] = ((q[:, h] @ np.swapaxes(k[:, h], -1, -2)) * M) @ v[:, h]
    np.testing.assert_allclose(orc.fwd_quadratic(q, k, v, decay), expect, rtol=1e-11, atol=1e-12)


def test_origin_equals_robust_identity():
    """App. C: kv_t (Algorithm 1) = lambda^-t * kvbar_t (Algorithm 2); outputs coincide."""
    Bt, H, N, D = 1, 2, 24, 6
    q, k, v = rnd((Bt, H, N, D), 31), rnd((Bt, H, N, D), 32), rnd((Bt, H, N, D), 33)
    decay = np.array([0.7, 0.95])
    o1, kv1 = orc.fwd_origin(q, k, v, decay)
    o2, kv2 = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    np.testing.assert_allclose(o1, o2, rtol=1e-9, atol=1e-12)
    for h in range(H):
        np.testing.assert_allclose(kv1[0, h], decay[h] ** (-N) * kv2[0, h], rtol=1e-9)


def test_origin_form_breaks_where_robust_does_not():
    """With the paper's strongest decay exp(-8), lambda^-t overflows fp64 before t = 100:
    Algorithm 1 yields non-finite outputs, Algorithm 2 stays finite (Sec. 3.3)."""
    Bt, H, N, D = 1, 1, 128, 4
    q, k, v = rnd((Bt, H, N, D), 41), rnd((Bt, H, N, D), 42), rnd((Bt, H, N, D), 43)
    decay = np.array([np.exp(-8.0)])
    o1, _ = orc.fwd_origin(q, k, v, decay)
    o2 = orc.fwd_recurrent(q, k, v, decay)
    assert not np.all(np.isfinite(o1))
    assert np.all(np.isfinite(o2))
    np.testing.assert_allclose(o2, orc.fwd_quadratic(q, k, v, decay), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("Br,Bc", [(4, 4), (8, 3), (5, 16), (64, 64)])
def test_paper_tiling_equals_definition(Br, Bc):
    """App. B Algorithm 3 with Br != Bc and ragged last tiles."""
    Bt, H, N, D = 1, 3, 37, 6
    q, k, v = rnd((Bt, H, N, D), 51), rnd((Bt, H, N, D), 52), rnd((Bt, H, N, D), 53)
    decay = np.array([0.5, 0.99, 1.0])
    np.testing.assert_allclose(orc.fwd_tiled(q, k, v, decay, Br, Bc),
                               orc.fwd_quadratic(q, k, v, decay), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("block", [1, 3, 16, 64, 100])
def test_block_form_equals_definition(block):
    Bt, H, N, D = 2, 3, 100, 8
    q, k, v = rnd((Bt, H, N, D), 61), rnd((Bt, H, N, D), 62), rnd((Bt, H, N, D), 63)
    decay = np.array([np.exp(-8.0), 0.9, 1.0])
    ref = brute_force_fwd(q[:, :, :24], k[:, :, :24], v[:, :, :24], decay)
    o, kv = orc.fwd_block(q, k, v, decay, block, return_state=True)
    o2, kv2 = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    np.testing.assert_allclose(o[:, :, :24], ref, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(o, orc.fwd_quadratic(q, k, v, decay), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(kv, kv2, rtol=1e-11, atol=1e-13)


def test_final_state_definition():
    """kv_out[i,j] = sum_s lambda^(N-1-s) k_s[i] v_s[j] (unrolled Algorithm 2)."""
    Bt, H, N, D = 1, 2, 19, 4
    k, v = rnd((Bt, H, N, D), 71), rnd((Bt, H, N, D), 72)
    q = rnd((Bt, H, N, D), 73)
    decay = np.array([0.6, 1.0])
    _, kv = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    for h in range(H):
        w = decay[h] ** (N - 1 - np.arange(N))
        expect = np.einsum("n,ni,nj->ij", w, k[0, h], v[0, h])
        np.testing.assert_allclose(kv[0, h], expect, rtol=1e-12, atol=1e-13)


def test_chunked_prefill():
    """fwd(N) == fwd(first part, state out) followed by fwd(second part, state in)."""
    Bt, H, N, D = 2, 2, 70, 6
    q, k, v = rnd((Bt, H, N, D), 81), rnd((Bt, H, N, D), 82), rnd((Bt, H, N, D), 83)
    decay = np.array([0.85, 0.3])
    full, kv_full = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    cut = 27
    o1, kv1 = orc.fwd_recurrent(q[:, :, :cut], k[:, :, :cut], v[:, :, :cut], decay, return_state=True)
    o2, kv2 = orc.fwd_recurrent(q[:, :, cut:], k[:, :, cut:], v[:, :, cut:], decay, kv_in=kv1,
                                return_state=True)
    np.testing.assert_allclose(np.concatenate([o1, o2], 2), full, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(kv2, kv_full, rtol=1e-12, atol=1e-13)
    o2b, kv2b = orc.fwd_block(q[:, :, cut:], k[:, :, cut:], v[:, :, cut:], decay, 16, kv_in=kv1,
                              return_state=True)
    np.testing.assert_allclose(o2b, o2, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(kv2b, kv2, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(full, orc.fwd_quadratic(q, k, v, decay), rtol=1e-11, atol=1e-13)


# --------------------------------------------------------------------------- backward


def test_bwd_finite_differences():
    """Central differences of L = <dO, O> evaluated with the quadratic forward.
    O is linear in each of Q, K, V, so central differences are exact up to rounding."""
    Bt, H, N, D = 1, 2, 11, 4
    q, k, v = rnd((Bt, H, N, D), 91), rnd((Bt, H, N, D), 92), rnd((Bt, H, N, D), 93)
    d_o = rnd((Bt, H, N, D), 94)
    decay = np.array([0.8, 0.2])
    dq, dk, dv = orc.bwd_quadratic(q, k, v, d_o, decay)
    eps = 1e-3

    def loss(qq, kk, vv):
        return float(np.sum(d_o * orc.fwd_quadratic(qq, kk, vv, decay)))

    for which, grad in ((0, dq), (1, dk), (2, dv)):
        num = np.zeros_like(q)
        for idx in np.ndindex(*q.shape):
            args_p = [q.copy(), k.copy(), v.copy()]
            args_m = [q.copy(), k.copy(), v.copy()]
            args_p[which][idx] += eps
            args_m[which][idx] -= eps
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * eps)
        assert orc.rel_l2(grad, num) < 1e-9, which


def test_bwd_matrix_form_with_numpy_matmul():
    """dV = A^T dO, dQ = dA K, dK = dA^T Q with dense A, dA built here (numpy matmul)."""
    Bt, H, N, D = 1, 2, 45, 7
    q, k, v = rnd((Bt, H, N, D), 101), rnd((Bt, H, N, D), 102), rnd((Bt, H, N, D), 103)
    d_o = rnd((Bt, H, N, D), 104)
    decay = np.array([0.93, 0.4])
    dq, dk, dv = orc.bwd_quadratic(q, k, v, d_o, decay)
    for h in range(H):
        M = dense_mask(decay[h], N)
        A = (q[0, h] @ k[0, h].T) * M
        dA = (d_o[0, h] @ v[0, h].T) * M
        np.testing.assert_allclose(dv[0, h], A.T @ d_o[0, h], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(dq[0, h], dA @ k[0, h], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(dk[0, h], dA.T @ q[0, h], rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("block", [1, 5, 16, 64])
def test_bwd_three_forms_agree(block):
    Bt, H, N, D = 2, 3, 75, 8
    q, k, v = rnd((Bt, H, N, D), 111), rnd((Bt, H, N, D), 112), rnd((Bt, H, N, D), 113)
    d_o = rnd((Bt, H, N, D), 114)
    decay = np.array([np.exp(-8.0), 0.97, 1.0])
    a = orc.bwd_quadratic(q, k, v, d_o, decay)
    b = orc.bwd_recurrent(q, k, v, d_o, decay)
    c = orc.bwd_block(q, k, v, d_o, decay, block)
    for x, y, z in zip(a, b, c):
        assert orc.max_rel_l2(y, x) < 1e-12
        assert orc.max_rel_l2(z, x) < 1e-12


def test_bwd_linearity_invariants():
    """O is linear in each of Q, K, V: <dQ,Q> = <dK,K> = <dV,V> = <dO,O> per (b,h)."""
    Bt, H, N, D = 2, 2, 64, 8
    q, k, v = rnd((Bt, H, N, D), 121), rnd((Bt, H, N, D), 122), rnd((Bt, H, N, D), 123)
    d_o = rnd((Bt, H, N, D), 124)
    decay = np.array([0.75, 0.999])
    o = orc.fwd_recurrent(q, k, v, decay)
    dq, dk, dv = orc.bwd_recurrent(q, k, v, d_o, decay)
    ref = np.sum(d_o * o, axis=(2, 3))
    for g, x in ((dq, q), (dk, k), (dv, v)):
        np.testing.assert_allclose(np.sum(g * x, axis=(2, 3)), ref, rtol=1e-10)


def test_bwd_probe_reads_back_masked_scores():
    """dO = e_t e_j^T  =>  dV[s, j] = A[t, s] for every s (and zero in other columns)."""
    Bt, H, N, D = 1, 1, 12, 3
    q, k, v = rnd((Bt, H, N, D), 131), rnd((Bt, H, N, D), 132), rnd((Bt, H, N, D), 133)
    lam = 0.6
    decay = np.array([lam])
    A = (q[0, 0] @ k[0, 0].T) * dense_mask(lam, N)
    for t, j in ((0, 0), (5, 1), (11, 2)):
        d_o = np.zeros((Bt, H, N, D))
        d_o[0, 0, t, j] = 1.0
        for f in (orc.bwd_quadratic, orc.bwd_recurrent):
            _, _, dv = f(q, k, v, d_o, decay)
            np.testing.assert_allclose(dv[0, 0, :, j], A[t], rtol=1e-12, atol=1e-14)
            mask = np.ones(D, bool)
            mask[j] = False
            assert np.all(dv[0, 0][:, mask] == 0)


# --------------------------------------------------------------------------- decode


def test_decode_steps_continue_a_prefix():
    """Decode steps from the prefix state reproduce the rows of one long forward."""
    Bt, H, N0, steps, D = 2, 3, 40, 25, 6
    N = N0 + steps
    q, k, v = rnd((Bt, H, N, D), 141), rnd((Bt, H, N, D), 142), rnd((Bt, H, N, D), 143)
    decay = np.array([0.9, 0.5, 1.0])
    full, kv_full = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    quad = orc.fwd_quadratic(q, k, v, decay)
    _, kv = orc.fwd_recurrent(q[:, :, :N0], k[:, :, :N0], v[:, :, :N0], decay, return_state=True)
    for t in range(N0, N):
        o, kv = orc.decode_step(q[:, :, t], k[:, :, t], v[:, :, t], kv, decay)
        np.testing.assert_allclose(o, quad[:, :, t], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(o, full[:, :, t], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(kv, kv_full, rtol=1e-12, atol=1e-13)


def test_decode_step_by_hand():
    """One step written out: kv' = lambda kv + k^T v, o = q kv' (update first, then read)."""
    Bt, H, D = 1, 2, 3
    q, k, v = rnd((Bt, H, D), 151), rnd((Bt, H, D), 152), rnd((Bt, H, D), 153)
    kv = rnd((Bt, H, D, D), 154)
    decay = np.array([0.3, 0.8])
    o, kv2 = orc.decode_step(q, k, v, kv, decay)
    for h in range(H):
        expect_kv = decay[h] * kv[0, h] + np.outer(k[0, h], v[0, h])
        np.testing.assert_allclose(kv2[0, h], expect_kv, rtol=1e-14)
        np.testing.assert_allclose(o[0, h], q[0, h] @ expect_kv, rtol=1e-13)


def test_bf16_inputs_are_widened_exactly():
    torch = pytest.importorskip("torch")
    g = torch.Generator().manual_seed(3)
    q = torch.randn(1, 1, 5, 4, generator=g).to(torch.bfloat16)
    k = torch.randn(1, 1, 5, 4, generator=g).to(torch.bfloat16)
    v = torch.randn(1, 1, 5, 4, generator=g).to(torch.bfloat16)
    decay = torch.tensor([0.5], dtype=torch.float32)
    a = orc.fwd_quadratic(q, k, v, decay)
    b = brute_force_fwd(q.double().numpy(), k.double().numpy(), v.double().numpy(), [0.5])
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-14)


def test_error_metric():
    x = np.ones((1, 2, 3, 4))
    y = x.copy()
    y[0, 1] *= 1.1
    assert abs(orc.rel_l2(y, x) - np.sqrt(12 * 0.01 / 24)) < 1e-12
    assert abs(orc.max_rel_l2(y, x) - 0.1) < 1e-12


# --------------------------------------------------------------------------- gated SimpleRMSNorm
# Sec. 3.1.2 Eq. 3 (O = Norm(.) (.) U) with the norm of Sec. 3.1.3, taken per head.


def _read_vectors(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                name, *vals = line.split()
                out[name] = np.array([float(x) for x in vals])
    return out


def test_gate_hand_example_golden():
    g = _read_vectors(os.path.join(GOLDEN, "hand_example_gate_d2.txt"))
    y = orc.gate_fwd(g["x"][None], g["u"][None])
    dx, du = orc.gate_bwd(g["x"][None], g["u"][None], g["dy"][None])
    np.testing.assert_allclose(y[0], g["y"], rtol=1e-14)
    np.testing.assert_allclose(dx[0], g["dx"], rtol=1e-13)
    np.testing.assert_allclose(du[0], g["du"], rtol=1e-14)


def test_gate_norm_is_sqrt_d_and_scale_invariant():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((7, 3, 11, 24))
    ones = np.ones_like(x)
    n = orc.gate_fwd(x, ones)
    np.testing.assert_allclose(np.linalg.norm(n, axis=-1), np.sqrt(24.0), rtol=1e-13)
    np.testing.assert_allclose(orc.gate_fwd(37.5 * x, ones), n, rtol=1e-13)
    np.testing.assert_allclose(orc.gate_fwd(-x, ones), -n, rtol=1e-13)


def test_gate_constant_row_and_library_norm():
    # a constant row c*1 normalises to sign(c)*1; in general x / (numpy's 2-norm / sqrt(d)) * u
    d = 16
    u = np.linspace(-2.0, 3.0, d)[None]
    np.testing.assert_allclose(orc.gate_fwd(np.full((1, d), -0.3), u), -u, rtol=1e-14)
    rng = np.random.default_rng(6)
    x, uu = rng.standard_normal((40, d)), rng.standard_normal((40, d))
    ref = x / (np.linalg.norm(x, axis=-1, keepdims=True) / np.sqrt(d)) * uu
    np.testing.assert_allclose(orc.gate_fwd(x, uu), ref, rtol=1e-13)


def test_gate_eps_enters_under_the_root():
    x = np.array([[0.0, 0.0, 0.0, 0.0], [1.0, -1.0, 1.0, -1.0]])
    u = np.array([[1.0, 2.0, 3.0, 4.0], [1.0, 2.0, 3.0, 4.0]])
    y = orc.gate_fwd(x, u, eps=3.0)          # second row: mean square 1, root of 1 + 3 = 2
    np.testing.assert_allclose(y, [[0, 0, 0, 0], [0.5, -1.0, 1.5, -2.0]], rtol=1e-15, atol=0)
    with np.errstate(all="ignore"):
        assert np.isnan(orc.gate_fwd(x, u)[0]).all()     # the printed formula: 0/0


@pytest.mark.parametrize("eps", [0.0, 1e-3])
def test_gate_bwd_finite_differences(eps):
    rng = np.random.default_rng(7)
    d = 12
    x, u, dy = (rng.standard_normal((5, d)) for _ in range(3))
    dx, du = orc.gate_bwd(x, u, dy, eps)
    h = 1e-6
    for arr, grad in ((x, dx), (u, du)):
        num = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            old = arr[idx]
            arr[idx] = old + h
            fp = float((orc.gate_fwd(x, u, eps) * dy).sum())
            arr[idx] = old - h
            fm = float((orc.gate_fwd(x, u, eps) * dy).sum())
            arr[idx] = old
            num[idx] = (fp - fm) / (2 * h)
        np.testing.assert_allclose(grad, num, rtol=2e-7, atol=2e-8)


def test_gate_bwd_invariants():
    # scale invariance of the norm (eps = 0) makes dx orthogonal to x; du is dy times the
    # normalised row; the map is linear in u, so <du, u> = <dy, y>
    rng = np.random.default_rng(8)
    x, u, dy = (rng.standard_normal((9, 32)) for _ in range(3))
    dx, du = orc.gate_bwd(x, u, dy)
    np.testing.assert_allclose((dx * x).sum(-1), 0.0, atol=1e-13)
    np.testing.assert_allclose(du, dy * orc.gate_fwd(x, np.ones_like(x)), rtol=1e-13)
    np.testing.assert_allclose((du * u).sum(), (dy * orc.gate_fwd(x, u)).sum(), rtol=1e-12)


def test_fwd_gated_composes_definition_and_gate():
    rng = np.random.default_rng(9)
    Bt, H, N, D = 1, 2, 9, 4
    q, k, v, u = (rng.standard_normal((Bt, H, N, D)) for _ in range(4))
    decay = np.array([0.9, 0.3])
    o, y = orc.fwd_gated(q, k, v, u, decay)
    np.testing.assert_allclose(o, brute_force_fwd(q, k, v, decay), rtol=1e-12, atol=1e-13)
    rms = np.sqrt((o ** 2).mean(-1, keepdims=True))
    np.testing.assert_allclose(y, o / rms * u, rtol=1e-12)
