"""Pins for the oracle's input side (swish of Eq. 2, LRPE-d of Eq. 1) and for the
variants of the recurrence and its gradients with a query/key width different from the
value width.  As in test_oracle_pins.py every function is checked against something other
than itself: loops written here, complex arithmetic, a hand-worked example, closed forms,
library routines and finite differences.

Runs without a GPU.
"""
import os

import numpy as np
import pytest
from scipy.special import expit

from oracle import ltn_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def loops_fwd_dkdv(q, k, v, decay):
    """O[t] = sum_{s<=t} lambda^(t-s) (q_t . k_s) v_s with q,k of width Dk and v of width Dv."""
    Bt, H, N, Dk = q.shape
    Dv = v.shape[3]
    o = np.zeros((Bt, H, N, Dv))
    for b in range(Bt):
        for h in range(H):
            for t in range(N):
                for s in range(t + 1):
                    w = 1.0
                    for _ in range(t - s):
                        w *= float(decay[h])
                    dot = sum(q[b, h, t, i] * k[b, h, s, i] for i in range(Dk))
                    for j in range(Dv):
                        o[b, h, t, j] += w * dot * v[b, h, s, j]
    return o


# ------------------------------------------------------------------ Dk != Dv


@pytest.mark.parametrize("N,Dk,Dv", [(1, 2, 1), (5, 6, 3), (9, 2, 5), (12, 8, 4)])
def test_dkdv_forward_vs_loops(N, Dk, Dv):
    Bt, H = 2, 3
    q, k, v = rnd((Bt, H, N, Dk), 1), rnd((Bt, H, N, Dk), 2), rnd((Bt, H, N, Dv), 3)
    decay = np.array([0.8, 0.0, 1.0])
    ref = loops_fwd_dkdv(q, k, v, decay)
    np.testing.assert_allclose(orc.fwd_quadratic_dkdv(q, k, v, decay), ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(orc.fwd_recurrent_dkdv(q, k, v, decay), ref, rtol=1e-12, atol=1e-13)


def test_dkdv_equal_widths_reduce_to_the_square_case():
    Bt, H, N, D = 2, 2, 33, 8
    q, k, v, g = (rnd((Bt, H, N, D), s) for s in (4, 5, 6, 7))
    decay = np.array([0.95, 0.4])
    o, kv = orc.fwd_recurrent_dkdv(q, k, v, decay, return_state=True)
    o0, kv0 = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    assert np.array_equal(o, o0) and np.array_equal(kv, kv0)
    for a, b in zip(orc.bwd_recurrent_dkdv(q, k, v, g, decay), orc.bwd_recurrent(q, k, v, g, decay)):
        assert np.array_equal(a, b)


def test_dkdv_zero_features_do_not_matter():
    # extra query/key features that are zero on one side change nothing
    Bt, H, N, Dk, Dv = 1, 2, 20, 5, 3
    q, k, v = rnd((Bt, H, N, Dk), 8), rnd((Bt, H, N, Dk), 9), rnd((Bt, H, N, Dv), 10)
    decay = np.array([0.9, 0.6])
    qp = np.concatenate([q, rnd((Bt, H, N, 4), 11)], axis=3)
    kp = np.concatenate([k, np.zeros((Bt, H, N, 4))], axis=3)
    np.testing.assert_allclose(orc.fwd_recurrent_dkdv(qp, kp, v, decay), orc.fwd_recurrent_dkdv(q, k, v, decay),
                               rtol=1e-13, atol=1e-14)


def test_dkdv_final_state_and_chunked_prefill():
    Bt, H, N, Dk, Dv = 2, 2, 37, 6, 4
    q, k, v = rnd((Bt, H, N, Dk), 12), rnd((Bt, H, N, Dk), 13), rnd((Bt, H, N, Dv), 14)
    decay = np.array([0.97, 0.5])
    o, kv = orc.fwd_recurrent_dkdv(q, k, v, decay, return_state=True)
    assert kv.shape == (Bt, H, Dk, Dv)
    for h in range(H):
        w = decay[h] ** (N - 1 - np.arange(N))
        ref = np.einsum("s,bsi,bsj->bij", w, k[:, h], v[:, h])     # rows: key feature, columns: value feature
        np.testing.assert_allclose(kv[:, h], ref, rtol=1e-12, atol=1e-13)
    c = 17
    o1, s1 = orc.fwd_recurrent_dkdv(q[:, :, :c], k[:, :, :c], v[:, :, :c], decay, return_state=True)
    o2, s2 = orc.fwd_recurrent_dkdv(q[:, :, c:], k[:, :, c:], v[:, :, c:], decay, kv_in=s1, return_state=True)
    np.testing.assert_allclose(np.concatenate([o1, o2], axis=2), o, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(s2, kv, rtol=1e-12, atol=1e-13)


def test_dkdv_backward_finite_differences_and_forms():
    Bt, H, N, Dk, Dv = 1, 2, 7, 4, 3
    q, k, v, g = rnd((Bt, H, N, Dk), 15), rnd((Bt, H, N, Dk), 16), rnd((Bt, H, N, Dv), 17), rnd((Bt, H, N, Dv), 18)
    decay = np.array([0.85, 0.3])

    def loss(q_, k_, v_):
        return float(np.sum(g * loops_fwd_dkdv(q_, k_, v_, decay)))

    grads = orc.bwd_quadratic_dkdv(q, k, v, g, decay)
    eps = 1e-6
    for which, (x, dx) in enumerate(zip((q, k, v), grads)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = [q, k, v]
            args_m = [q, k, v]
            args_p[which], args_m[which] = xp, xm
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * eps)
        np.testing.assert_allclose(dx, num, rtol=1e-7, atol=1e-8)
    for a, b in zip(orc.bwd_recurrent_dkdv(q, k, v, g, decay), grads):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)


def test_dkdv_backward_linearity_invariants():
    # O is linear in each of Q, K, V: <dX, X> = <dO, O> for each of them
    Bt, H, N, Dk, Dv = 2, 2, 50, 8, 4
    q, k, v, g = rnd((Bt, H, N, Dk), 19), rnd((Bt, H, N, Dk), 20), rnd((Bt, H, N, Dv), 21), rnd((Bt, H, N, Dv), 22)
    decay = np.array([0.99, 0.7])
    o = orc.fwd_recurrent_dkdv(q, k, v, decay)
    dq, dk, dv = orc.bwd_recurrent_dkdv(q, k, v, g, decay)
    ref = np.sum(g * o, axis=(2, 3))
    for dx, x in ((dq, q), (dk, k), (dv, v)):
        np.testing.assert_allclose(np.sum(dx * x, axis=(2, 3)), ref, rtol=1e-11)


def test_dkdv_decode_by_hand_and_continuation():
    # Dk = 2, Dv = 1: kv = [[1],[2]], lambda = 1/2, k = (1,-1), v = 3 -> kv = [[3.5],[-2]]; q = (2,1) -> o = 5
    o, kv = orc.decode_step_dkdv(np.array([[[2.0, 1.0]]]), np.array([[[1.0, -1.0]]]), np.array([[[3.0]]]),
                                 np.array([[[[1.0], [2.0]]]]), np.array([0.5]))
    assert np.array_equal(kv, np.array([[[[3.5], [-2.0]]]])) and np.array_equal(o, np.array([[[5.0]]]))
    Bt, H, N, Dk, Dv = 2, 2, 12, 6, 3
    q, k, v = rnd((Bt, H, N, Dk), 23), rnd((Bt, H, N, Dk), 24), rnd((Bt, H, N, Dv), 25)
    decay = np.array([0.9, 0.2])
    ref, ref_state = orc.fwd_recurrent_dkdv(q, k, v, decay, return_state=True)
    _, state = orc.fwd_recurrent_dkdv(q[:, :, :5], k[:, :, :5], v[:, :, :5], decay, return_state=True)
    for t in range(5, N):
        o, state = orc.decode_step_dkdv(q[:, :, t], k[:, :, t], v[:, :, t], state, decay)
        np.testing.assert_allclose(o, ref[:, :, t], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(state, ref_state, rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ swish (Eq. 2)


def test_swish_values_and_library_sigmoid():
    x = np.concatenate([np.linspace(-30, 30, 241), [0.0, 1e-8, -1e-8, 700.0, -700.0]]).reshape(1, 1, -1, 1)
    y = orc.prologue_fwd(x, None, act=True)
    np.testing.assert_allclose(y, x * expit(x), rtol=1e-14, atol=1e-300)
    assert y[0, 0, 241, 0] == 0.0                                     # phi(0) = 0
    np.testing.assert_allclose(y - orc.prologue_fwd(-x, None, act=True), x, rtol=1e-13, atol=1e-15)  # phi(x) - phi(-x) = x
    assert y[0, 0, 244, 0] == 700.0 and abs(y[0, 0, 245, 0]) < 1e-290  # identity far right, zero far left
    # the minimum of x sigma(x): value -0.27846454276107..., where 1 + x (1 - sigma(x)) = 0
    xs = np.linspace(-1.3, -1.25, 50001).reshape(1, 1, -1, 1)
    ys = orc.prologue_fwd(xs, None, act=True)
    assert abs(ys.min() + 0.27846454276107) < 1e-10
    # act = False passes values through
    assert np.array_equal(orc.prologue_fwd(x, None, act=False), x)


# ------------------------------------------------------------------ LRPE-d (Eq. 1)


def read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *nums = line.split()
            vals[key] = np.array([float(x) for x in nums])
    return vals


def test_lrpe_hand_example_golden():
    gld = read_golden("hand_example_lrpe_d1.txt")
    theta = np.array([[gld["theta_over_pi"][0] * np.pi]])
    lam = gld["lambda"]
    q, k, v = (gld[n].reshape(1, 1, 4, 1) for n in ("q", "k", "v"))
    np.testing.assert_allclose(orc.lrpe_fwd_quadratic(q, k, v, lam, theta).ravel(), gld["o"], rtol=0, atol=1e-15)
    qe = orc.prologue_fwd(q, theta, act=False)
    np.testing.assert_allclose(qe[0, 0, :, 0], gld["qc"], atol=1e-15)
    np.testing.assert_allclose(qe[0, 0, :, 1], gld["qs"], atol=1e-15)
    ke = orc.prologue_fwd(k, theta, act=False)
    np.testing.assert_allclose(orc.fwd_recurrent_dkdv(qe, ke, v, lam).ravel(), gld["o"], rtol=0, atol=1e-15)


def complex_scores(q, k, theta_h, lam):
    """a[t,s] = Re( sum_d q_t[d] k_s[d] exp(i theta_d (t-s)) ) lambda^(t-s), by a complex matrix
    product of (q_t e^{i theta t}) with (k_s e^{-i theta s})."""
    N = q.shape[0]
    pos = np.arange(N)[:, None]
    qt = q * np.exp(1j * theta_h[None, :] * pos)
    ks = k * np.exp(-1j * theta_h[None, :] * pos)
    a = (qt @ ks.T).real
    d = pos - pos.T
    m = np.where(d >= 0, float(lam) ** np.maximum(d, 0), 0.0)
    return a * m


def test_lrpe_definition_vs_complex_arithmetic():
    Bt, H, N, D = 2, 3, 40, 6
    q, k, v = rnd((Bt, H, N, D), 30), rnd((Bt, H, N, D), 31), rnd((Bt, H, N, D), 32)
    decay = np.array([0.9, 0.5, 1.0])
    theta = np.random.default_rng(33).uniform(0.0, 2.0, (H, D))
    o = orc.lrpe_fwd_quadratic(q, k, v, decay, theta)
    for b in range(Bt):
        for h in range(H):
            ref = complex_scores(q[b, h], k[b, h], theta[h], decay[h]) @ v[b, h]
            np.testing.assert_allclose(o[b, h], ref, rtol=1e-11, atol=1e-12)


def test_lrpe_zero_angle_is_plain_attention():
    Bt, H, N, D = 1, 2, 25, 5
    q, k, v = rnd((Bt, H, N, D), 34), rnd((Bt, H, N, D), 35), rnd((Bt, H, N, D), 36)
    decay = np.array([0.8, 0.99])
    np.testing.assert_allclose(orc.lrpe_fwd_quadratic(q, k, v, decay, np.zeros((H, D))),
                               orc.fwd_quadratic(q, k, v, decay), rtol=1e-14, atol=1e-15)
    # and the expansion at zero angle is [z | 0]
    y = orc.prologue_fwd(q, np.zeros((H, D)), act=False, pos0=7)
    assert np.array_equal(y[..., :D], q) and not y[..., D:].any()


@pytest.mark.parametrize("pos0", [0, 5, 100000])
def test_lrpe_expansion_reproduces_the_definition_at_any_offset(pos0):
    # the separable form: queries and keys expanded at absolute positions, then the plain
    # recurrence with Dk = 2D; only position differences matter
    Bt, H, N, D = 2, 2, 30, 4
    q, k, v = rnd((Bt, H, N, D), 37), rnd((Bt, H, N, D), 38), rnd((Bt, H, N, D), 39)
    decay = np.array([0.93, 0.6])
    theta = np.random.default_rng(40).uniform(0.0, 1.0, (H, D))
    ref = orc.lrpe_fwd_quadratic(q, k, v, decay, theta)
    qe = orc.prologue_fwd(q, theta, act=False, pos0=pos0)
    ke = orc.prologue_fwd(k, theta, act=False, pos0=pos0)
    assert qe.shape == (Bt, H, N, 2 * D)
    np.testing.assert_allclose(orc.fwd_recurrent_dkdv(qe, ke, v, decay), ref, rtol=1e-9, atol=1e-10)


def test_lrpe_expansion_layout_and_norm():
    Bt, H, N, D = 2, 3, 16, 5
    x = rnd((Bt, H, N, D), 41)
    theta = np.random.default_rng(42).uniform(0.0, 3.0, (H, D))
    pos0 = 11
    y = orc.prologue_fwd(x, theta, act=True, pos0=pos0)
    z = x * expit(x)
    p = (pos0 + np.arange(N))[None, None, :, None]
    np.testing.assert_allclose(y[..., :D], z * np.cos(theta[None, :, None, :] * p), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(y[..., D:], z * np.sin(theta[None, :, None, :] * p), rtol=1e-12, atol=1e-14)
    # the phase does not change a row's norm (the remark of Sec. 3.3)
    np.testing.assert_allclose(np.linalg.norm(y, axis=3), np.linalg.norm(z, axis=3), rtol=1e-13)


@pytest.mark.parametrize("act,with_theta", [(True, True), (False, True), (True, False)])
def test_prologue_bwd_finite_differences(act, with_theta):
    Bt, H, N, D = 2, 2, 6, 3
    pos0 = 3
    x = rnd((Bt, H, N, D), 43)
    theta = np.random.default_rng(44).uniform(0.1, 1.5, (H, D)) if with_theta else None
    g = rnd((Bt, H, N, 2 * D if with_theta else D), 45)

    def loss(x_, th_):
        return float(np.sum(g * orc.prologue_fwd(x_, th_, act=act, pos0=pos0)))

    dx, dth = orc.prologue_bwd(x, g, theta, act=act, pos0=pos0)
    eps = 1e-6
    num = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps
        xm[idx] -= eps
        num[idx] = (loss(xp, theta) - loss(xm, theta)) / (2 * eps)
    np.testing.assert_allclose(dx, num, rtol=1e-7, atol=1e-8)
    if not with_theta:
        assert dth is None
        return
    numt = np.zeros_like(theta)
    for h in range(H):
        for d in range(D):
            tp, tm = theta.copy(), theta.copy()
            tp[h, d] += eps
            tm[h, d] -= eps
            numt[h, d] = (loss(x, tp) - loss(x, tm)) / (2 * eps)
    np.testing.assert_allclose(dth, numt, rtol=1e-6, atol=1e-7)


def test_lrpe_end_to_end_gradient_of_the_definition():
    # chain rule through expansion and recurrence against finite differences of Eq. 1 itself
    Bt, H, N, D = 1, 2, 6, 2
    q, k, v, g = (rnd((Bt, H, N, D), s) for s in (46, 47, 48, 49))
    decay = np.array([0.9, 0.5])
    theta = np.random.default_rng(50).uniform(0.1, 1.0, (H, D))

    def loss(q_, k_, th_):
        return float(np.sum(g * orc.lrpe_fwd_quadratic(q_, k_, v, decay, th_)))

    qe, ke = orc.prologue_fwd(q, theta, act=False), orc.prologue_fwd(k, theta, act=False)
    dqe, dke, _ = orc.bwd_recurrent_dkdv(qe, ke, v, g, decay)
    dq, dth_q = orc.prologue_bwd(q, dqe, theta, act=False)
    dk, dth_k = orc.prologue_bwd(k, dke, theta, act=False)
    eps = 1e-6
    for x, dx, which in ((q, dq, 0), (k, dk, 1)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            num[idx] = ((loss(xp, k, theta) - loss(xm, k, theta)) if which == 0
                        else (loss(q, xp, theta) - loss(q, xm, theta))) / (2 * eps)
        np.testing.assert_allclose(dx, num, rtol=1e-6, atol=1e-8)
    numt = np.zeros_like(theta)
    for h in range(H):
        for d in range(D):
            tp, tm = theta.copy(), theta.copy()
            tp[h, d] += eps
            tm[h, d] -= eps
            numt[h, d] = (loss(q, k, tp) - loss(q, k, tm)) / (2 * eps)
    np.testing.assert_allclose(dth_q + dth_k, numt, rtol=1e-6, atol=1e-7)
