"""GPU parity of the input side of the token mixer -- swish (Sec. 3.1.2 Eq. 2) and the LRPE-d
expansion (Sec. 3.1.1 Eq. 1) -- and of the attention kernels behind it, whose queries and
keys are twice as wide as the values; all through the C ABI against the fp64 oracle on the
same seeded inputs."""
import numpy as np
import pytest
import torch

import paper_2307_14995_amd as ltn
from paper_2307_14995_amd import synth
from oracle import ltn_oracle as orc
from _helpers import TOL_ROW, check, check_rows, dev, force_plan, gpu, mixed_decay

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-4, torch.bfloat16: 1e-2}
SHAPES = [(256, 128), (128, 64)]


# ------------------------------------------------------------------ attention, Dk = 2 Dv


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("Dk,Dv", SHAPES)
@pytest.mark.parametrize("N", [1, 63, 64, 65, 200, 517])
def test_dkdv_forward_ragged(dtype, Dk, Dv, N):
    Bt, H = 1, 3
    q, k, v = synth.make_qkv_dkdv(Bt, H, N, Dk, Dv, dtype, 500 + N)
    decay = mixed_decay(H)
    o, kv = ltn.ltn_attn_fwd_dkdv(*gpu(q, k, v, decay), return_state=True)
    ref, ref_kv = orc.fwd_recurrent_dkdv(q, k, v, decay, return_state=True)
    assert o.shape == v.shape and kv.shape == (Bt, H, Dk, Dv)
    check("o", o, ref, TOL[dtype])
    check("kv_out", kv, ref_kv, TOL[dtype])


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("Dk,Dv", SHAPES)
def test_dkdv_state_in_and_chunked_prefill(dtype, Dk, Dv):
    Bt, H, N, cut = 2, 4, 330, 130
    q, k, v = synth.make_qkv_dkdv(Bt, H, N, Dk, Dv, dtype, 520)
    decay = synth.decay_bench_rule(H)
    g = torch.Generator().manual_seed(521)
    kv0 = torch.randn(Bt, H, Dk, Dv, generator=g)
    ref, ref_kv = orc.fwd_recurrent_dkdv(q, k, v, decay, kv_in=kv0, return_state=True)
    qd, kd, vd, dd, kv0d = gpu(q, k, v, decay, kv0)
    o, kv = ltn.ltn_attn_fwd_dkdv(qd, kd, vd, dd, kv_in=kv0d, return_state=True)
    check("o", o, ref, TOL[dtype])
    check("kv", kv, ref_kv, TOL[dtype])
    o1, s1 = ltn.ltn_attn_fwd_dkdv(qd[:, :, :cut].contiguous(), kd[:, :, :cut].contiguous(),
                                   vd[:, :, :cut].contiguous(), dd, kv_in=kv0d, return_state=True)
    o2, s2 = ltn.ltn_attn_fwd_dkdv(qd[:, :, cut:].contiguous(), kd[:, :, cut:].contiguous(),
                                   vd[:, :, cut:].contiguous(), dd, kv_in=s1, return_state=True)
    check("chunked o", torch.cat([o1, o2], dim=2), ref, TOL[dtype])
    check("chunked kv", s2, ref_kv, TOL[dtype])


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("Dk,Dv", SHAPES)
@pytest.mark.parametrize("N", [1, 65, 300])
def test_dkdv_backward(dtype, Dk, Dv, N):
    Bt, H = 1, 3
    q, k, v = synth.make_qkv_dkdv(Bt, H, N, Dk, Dv, dtype, 540 + N)
    d_o = synth.make_do(Bt, H, N, Dv, dtype, 540 + N)
    decay = mixed_decay(H)
    dq, dk, dv = ltn.ltn_attn_bwd_dkdv(*gpu(q, k, v, d_o, decay))
    rq, rk, rv = orc.bwd_recurrent_dkdv(q, k, v, d_o, decay)
    assert dq.shape == q.shape and dk.shape == k.shape and dv.shape == v.shape
    check("dq", dq, rq, TOL[dtype])
    check("dk", dk, rk, TOL[dtype])
    check("dv", dv, rv, TOL[dtype])


@pytest.mark.parametrize("Dk,Dv", SHAPES)
@pytest.mark.parametrize("Bt,H", [(1, 2), (4, 24), (10, 30)])
def test_dkdv_every_column_split(Dk, Dv, Bt, H):
    # the number of chains decides how many value columns a workgroup takes: 2, 96 and 300
    # chains reach every slice width of the forward and of both backward launches
    N = 130
    for dtype in (torch.bfloat16, torch.float32):
        q, k, v = synth.make_qkv_dkdv(Bt, H, N, Dk, Dv, dtype, 560 + H)
        d_o = synth.make_do(Bt, H, N, Dv, dtype, 560 + H)
        decay = synth.decay_bench_rule(H)
        qd, kd, vd, gd, dd = gpu(q, k, v, d_o, decay)
        check("o", ltn.ltn_attn_fwd_dkdv(qd, kd, vd, dd), orc.fwd_recurrent_dkdv(q, k, v, decay), TOL[dtype])
        for name, got, ref in zip(("dq", "dk", "dv"), ltn.ltn_attn_bwd_dkdv(qd, kd, vd, gd, dd),
                                  orc.bwd_recurrent_dkdv(q, k, v, d_o, decay)):
            check(name, got, ref, TOL[dtype])


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("Dk,Dv", SHAPES)
def test_dkdv_decode_continues_a_prefix(dtype, Dk, Dv):
    Bt, H, N0, S = 2, 3, 100, 9
    q, k, v = synth.make_qkv_dkdv(Bt, H, N0 + S, Dk, Dv, dtype, 580)
    decay = mixed_decay(H)
    ref, ref_kv = orc.fwd_recurrent_dkdv(q, k, v, decay, return_state=True)
    qd, kd, vd, dd = gpu(q, k, v, decay)
    _, kv = ltn.ltn_attn_fwd_dkdv(qd[:, :, :N0].contiguous(), kd[:, :, :N0].contiguous(),
                                  vd[:, :, :N0].contiguous(), dd, return_state=True)
    # four tokens in one call, then the rest one at a time
    o_a = ltn.ltn_attn_decode_steps_dkdv(qd[:, :, N0:N0 + 4].contiguous(), kd[:, :, N0:N0 + 4].contiguous(),
                                         vd[:, :, N0:N0 + 4].contiguous(), kv, dd)
    outs = [o_a]
    for t in range(N0 + 4, N0 + S):
        outs.append(ltn.ltn_attn_decode_steps_dkdv(qd[:, :, t:t + 1].contiguous(), kd[:, :, t:t + 1].contiguous(),
                                                   vd[:, :, t:t + 1].contiguous(), kv, dd))
    check("decode o", torch.cat(outs, dim=2), ref[:, :, N0:], TOL[dtype])
    check("decode kv", kv, ref_kv, TOL[dtype])


def test_dkdv_empty_and_errors():
    H, Dk, Dv = 2, 256, 128
    decay = synth.decay_bench_rule(H).to(dev())
    kv0 = torch.randn(1, H, Dk, Dv, device=dev())
    z = torch.zeros(1, H, 0, Dk, dtype=torch.bfloat16, device=dev())
    zv = torch.zeros(1, H, 0, Dv, dtype=torch.bfloat16, device=dev())
    o, kv = ltn.ltn_attn_fwd_dkdv(z, z, zv, decay, kv_in=kv0, return_state=True)
    assert o.shape == (1, H, 0, Dv) and torch.equal(kv, kv0)
    a = torch.zeros(1, H, 8, 128, dtype=torch.bfloat16, device=dev())
    with pytest.raises(ltn.LtnError):
        ltn.ltn_attn_fwd_dkdv(a, a.clone(), a.clone(), decay)          # equal widths: not this entry point
    with pytest.raises(ltn.LtnError):
        ltn.ltn_attn_fwd_dkdv(a, a.clone(), a[..., :32].contiguous(), decay)


@pytest.mark.parametrize("Dk,Dv", SHAPES)
@pytest.mark.parametrize("N,segs", [(130, 2), (517, 3), (1000, 5)])
def test_dkdv_segmented_forward_backward(Dk, Dv, N, segs):
    """Chains cut into segments (forced): state-only sweep, scan over [Dk x Dv] states, per-segment
    pass; with an initial state, the final state, and all three gradients."""
    Bt, H = 1, 3
    dtype = torch.bfloat16
    q, k, v = synth.make_qkv_dkdv(Bt, H, N, Dk, Dv, dtype, 620 + N)
    d_o = synth.make_do(Bt, H, N, Dv, dtype, 620 + N)
    kv0 = torch.randn(Bt, H, Dk, Dv, generator=torch.Generator().manual_seed(N)) * 0.1
    decay = mixed_decay(H)
    ref, kv_ref = orc.fwd_recurrent_dkdv(q, k, v, decay, kv_in=kv0, return_state=True)
    refs = orc.bwd_recurrent_dkdv(q, k, v, d_o, decay)
    with force_plan(segs=segs):
        assert ltn.ltn_attn_workspace_bytes_dkdv(Bt, H, N, Dk, Dv, dtype, 0) > 0
        assert ltn.ltn_attn_workspace_bytes_dkdv(Bt, H, N, Dk, Dv, dtype, 1) > 0
        o, kv = ltn.ltn_attn_fwd_dkdv(*gpu(q, k, v, decay), kv_in=kv0.to(dev()), return_state=True)
        o2 = ltn.ltn_attn_fwd_dkdv(*gpu(q, k, v, decay), kv_in=kv0.to(dev()))       # final state not requested
        grads = ltn.ltn_attn_bwd_dkdv(*gpu(q, k, v, d_o, decay))
    check("o", o, ref, 1e-2)
    check("kv", kv, kv_ref, 1e-2)
    assert torch.equal(o2, o)
    for name, got, r in zip(("dq", "dk", "dv"), grads, refs):
        check(name, got, r, 1e-2)


def _random_cases_dkdv(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        Dk, Dv = SHAPES[int(rng.integers(0, len(SHAPES)))]
        Bt, H = int(rng.integers(1, 4)), int(rng.integers(1, 13))       # the chain count decides the slice width
        N = int(rng.choice([rng.integers(1, 64), rng.integers(64, 400), rng.integers(400, 1200)]))
        dtype = torch.bfloat16 if rng.integers(0, 3) else torch.float32
        segs = int(rng.choice([1, 2, 3, 6])) if dtype == torch.bfloat16 else 0
        cases.append((i, Bt, H, N, Dk, Dv, dtype, segs))
    return cases


@pytest.mark.parametrize("case", _random_cases_dkdv(12, 2027),
                         ids=lambda c: "B%dH%dN%dDk%dDv%d%sseg%d" % (c[1:6] + (str(c[6]).split(".")[-1],) + c[7:]))
def test_dkdv_seeded_shape_sweep(case):
    """Unequal widths on seeded odd shapes, both dtypes, segment count forced (bf16)."""
    i, Bt, H, N, Dk, Dv, dtype, segs = case
    tol = TOL[dtype]
    q, k, v = synth.make_qkv_dkdv(Bt, H, N, Dk, Dv, dtype, 660 + i)
    d_o = synth.make_do(Bt, H, N, Dv, dtype, 660 + i)
    kv0 = torch.randn(Bt, H, Dk, Dv, generator=torch.Generator().manual_seed(90 + i)) * 0.1
    decay = torch.rand(H, generator=torch.Generator().manual_seed(1300 + i))
    decay[0] = 1.0
    ref, kv_ref = orc.fwd_recurrent_dkdv(q, k, v, decay, kv_in=kv0, return_state=True)
    refs = orc.bwd_recurrent_dkdv(q, k, v, d_o, decay)
    with force_plan(segs=segs):
        o, kv = ltn.ltn_attn_fwd_dkdv(*gpu(q, k, v, decay), kv_in=kv0.to(dev()), return_state=True)
        grads = ltn.ltn_attn_bwd_dkdv(*gpu(q, k, v, d_o, decay))
    check("o", o, ref, tol)
    check("kv", kv, kv_ref, tol)
    for name, got, r in zip(("dq", "dk", "dv"), grads, refs):
        check(name, got, r, tol)


def test_dkdv_few_long_chains_are_cut_into_segments_by_default():
    Bt, H, N, Dk, Dv = 1, 4, 4096 + 70, 256, 128         # 4 chains x 2 slices: cut 8 ways by the library's own rule
    dtype = torch.bfloat16
    assert ltn.ltn_attn_workspace_bytes_dkdv(Bt, H, N, Dk, Dv, dtype, 0) == 8 * Bt * H * Dk * Dv * 4
    q, k, v = synth.make_qkv_dkdv(Bt, H, N, Dk, Dv, dtype, 640)
    d_o = synth.make_do(Bt, H, N, Dv, dtype, 640)
    decay = synth.decay_bench_rule(H)
    o, kv = ltn.ltn_attn_fwd_dkdv(*gpu(q, k, v, decay), return_state=True)
    ref, kv_ref = orc.fwd_recurrent_dkdv(q, k, v, decay, return_state=True)
    check("o", o, ref, 1e-2)
    check_rows("o rows", o, ref, TOL_ROW[dtype])
    check("kv", kv, kv_ref, 1e-2)
    for name, got, r in zip(("dq", "dk", "dv"), ltn.ltn_attn_bwd_dkdv(*gpu(q, k, v, d_o, decay)),
                            orc.bwd_recurrent_dkdv(q, k, v, d_o, decay)):
        check(name, got, r, 1e-2)
        check_rows(name + " rows", got, r, TOL_ROW[dtype])


def test_dkdv_full_size_every_chain():
    # first-layer shape of the 7B-sized model, the launch configuration the report times: every
    # chain against the oracle (batch entry by batch entry), slice by slice and token by token
    Bt, H, N, Dk, Dv = 4, 32, 8192, 256, 128
    dtype = torch.bfloat16
    q, k, v = synth.make_qkv_dkdv(Bt, H, N, Dk, Dv, dtype, 600)
    d_o = synth.make_do(Bt, H, N, Dv, dtype, 600)
    decay = synth.decay_bench_rule(H)
    qd, kd, vd, gd, dd = gpu(q, k, v, d_o, decay)
    o = ltn.ltn_attn_fwd_dkdv(qd, kd, vd, dd).cpu()
    grads = tuple(x.cpu() for x in ltn.ltn_attn_bwd_dkdv(qd, kd, vd, gd, dd))
    for b in range(Bt):
        sl = slice(b, b + 1)
        refs = (orc.fwd_recurrent_dkdv(q[sl], k[sl], v[sl], decay),) + tuple(
            orc.bwd_recurrent_dkdv(q[sl], k[sl], v[sl], d_o[sl], decay))
        for name, got, r in zip(("o", "dq", "dk", "dv"), (o,) + grads, refs):
            check(f"{name}[{b}]", got[sl], r, TOL[dtype])
            check_rows(f"{name}[{b}] rows", got[sl], r, TOL_ROW[dtype])


# ------------------------------------------------------------------ swish and the expansion


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("act,with_theta", [(True, True), (False, True), (True, False)])
@pytest.mark.parametrize("pos0", [0, 1000003])
def test_prologue_forward_backward(dtype, D, act, with_theta, pos0):
    Bt, H, N = 2, 3, 203                                 # three full 64-token chunks and a ragged one
    x = synth.make_preact(Bt, H, N, D, dtype, 620 + D)
    theta = synth.make_theta(H, D, 621) if with_theta else None
    W = 2 * D if with_theta else D
    g = torch.Generator().manual_seed(622 + D)
    dy = torch.randn(Bt, H, N, W, generator=g).to(dtype)
    xd, thd, dyd = gpu(x, theta, dy)
    y = ltn.ltn_prologue_fwd(xd, thd, act=act, pos0=pos0)
    assert y.shape == (Bt, H, N, W)
    check("y", y, orc.prologue_fwd(x, theta, act=act, pos0=pos0), TOL[dtype])
    dx, dth = ltn.ltn_prologue_bwd(xd, dyd, thd, act=act, pos0=pos0)
    rdx, rdth = orc.prologue_bwd(x, dy, theta, act=act, pos0=pos0)
    check("dx", dx, rdx, TOL[dtype])
    if with_theta:
        assert orc.rel_l2(dth, rdth) <= TOL[dtype], orc.rel_l2(dth, rdth)
        # reproducible: the sum over tokens is taken in a fixed order
        _, dth2 = ltn.ltn_prologue_bwd(xd, dyd, thd, act=act, pos0=pos0)
        assert torch.equal(dth, dth2)
        # and it can be skipped
        dx3, none = ltn.ltn_prologue_bwd(xd, dyd, thd, act=act, pos0=pos0, want_dtheta=False)
        assert none is None and torch.equal(dx3, dx)
    else:
        assert dth is None


def test_prologue_elementwise_extremes():
    # swish far from the origin, zero angles, and a single token
    D, H = 128, 1
    vals = torch.tensor([0.0, -0.0, 1e-6, -1e-6, 1.0, -1.2785, 20.0, -20.0, 88.0, -88.0, 200.0, -200.0, 3e4, -3e4])
    x = vals.repeat(D // 2 + 1)[:D].reshape(1, H, 1, D).contiguous()
    theta = torch.zeros(H, D)
    for dtype in (torch.float32, torch.bfloat16):
        xs = x.to(dtype)
        y = ltn.ltn_prologue_fwd(xs.to(dev()), theta.to(dev()), act=True, pos0=12345)
        ref = orc.prologue_fwd(xs, theta, act=True, pos0=12345)
        assert torch.isfinite(y.float()).all()
        assert not y[..., D:].float().any()                  # sin(0) = 0 exactly
        np.testing.assert_allclose(y.double().cpu().numpy(), ref, rtol=1e-2 if dtype == torch.bfloat16 else 2e-6,
                                   atol=1e-30)
        dy = torch.ones(1, H, 1, 2 * D, dtype=dtype)
        dx, _ = ltn.ltn_prologue_bwd(xs.to(dev()), dy.to(dev()), theta.to(dev()), act=True, pos0=12345)
        rdx, _ = orc.prologue_bwd(xs, dy, theta, act=True, pos0=12345)
        assert torch.isfinite(dx.float()).all()
        np.testing.assert_allclose(dx.double().cpu().numpy(), rdx, rtol=1e-2 if dtype == torch.bfloat16 else 2e-6,
                                   atol=1e-6)


def test_prologue_phase_accuracy_at_large_positions():
    # x = 1 without activation writes [cos | sin](theta p) themselves: the angle must keep its
    # phase at positions far beyond what an fp32 product theta * p could resolve
    H, D, N = 3, 128, 1024
    theta = synth.make_theta(H, D, 630)
    theta[1] = torch.rand(D, generator=torch.Generator().manual_seed(631)) * 6.0
    x = torch.ones(1, H, N, D)
    for pos0 in (0, 1000003, 10 ** 9):
        y = ltn.ltn_prologue_fwd(x.to(dev()), theta.to(dev()), act=False, pos0=pos0)
        ref = orc.prologue_fwd(x, theta, act=False, pos0=pos0)
        assert np.abs(y.double().cpu().numpy() - ref).max() <= 2e-6


def test_prologue_empty():
    H, D = 2, 64
    theta = synth.make_theta(H, D, 1).to(dev())
    x = torch.zeros(1, H, 0, D, dtype=torch.bfloat16, device=dev())
    assert ltn.ltn_prologue_fwd(x, theta).shape == (1, H, 0, 2 * D)
    dy = torch.zeros(1, H, 0, 2 * D, dtype=torch.bfloat16, device=dev())
    dx, dth = ltn.ltn_prologue_bwd(x, dy, theta)
    assert dx.shape == x.shape and dth.shape == (H, D) and not dth.any()


# ------------------------------------------------------------------ end to end: Eq. 1 as printed


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("D", [64, 128])
def test_lrpe_attention_matches_the_definition(dtype, D):
    # swish + expansion + attention on the GPU against the quadratic evaluation of Eq. 1's
    # real part; a position offset must not matter
    Bt, H, N = 2, 3, 300
    xq = synth.make_preact(Bt, H, N, D, dtype, 640, 0)
    xk = synth.make_preact(Bt, H, N, D, dtype, 640, 1)
    _, _, v = synth.make_qkv(Bt, H, N, D, dtype, 640)
    theta = synth.make_theta(H, D, 641)
    decay = mixed_decay(H)
    zq, zk = orc.prologue_fwd(xq, None, act=True), orc.prologue_fwd(xk, None, act=True)
    ref = orc.lrpe_fwd_quadratic(zq, zk, v, decay, theta)
    xqd, xkd, vd, thd, dd = gpu(xq, xk, v, theta, decay)
    for pos0 in (0, 4096):
        qe = ltn.ltn_prologue_fwd(xqd, thd, act=True, pos0=pos0)
        ke = ltn.ltn_prologue_fwd(xkd, thd, act=True, pos0=pos0)
        check(f"o (pos0={pos0})", ltn.ltn_attn_fwd_dkdv(qe, ke, vd, dd), ref, TOL[dtype])


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_lrpe_training_chain_gradients(dtype):
    # forward and backward of (swish, expansion, attention) chained on the GPU against the
    # same chain in the oracle: gradients with respect to the pre-activations and the angles
    Bt, H, N, D = 2, 2, 260, 128
    xq = synth.make_preact(Bt, H, N, D, dtype, 660, 0)
    xk = synth.make_preact(Bt, H, N, D, dtype, 660, 1)
    _, _, v = synth.make_qkv(Bt, H, N, D, dtype, 660)
    d_o = synth.make_do(Bt, H, N, D, dtype, 660)
    theta = synth.make_theta(H, D, 661)
    decay = synth.decay_bench_rule(H)
    # oracle chain in fp64 from the same inputs
    qe_r, ke_r = orc.prologue_fwd(xq, theta), orc.prologue_fwd(xk, theta)
    dqe_r, dke_r, dv_r = orc.bwd_recurrent_dkdv(qe_r, ke_r, v, d_o, decay)
    dxq_r, dthq_r = orc.prologue_bwd(xq, dqe_r, theta)
    dxk_r, dthk_r = orc.prologue_bwd(xk, dke_r, theta)
    # GPU chain
    xqd, xkd, vd, gd, thd, dd = gpu(xq, xk, v, d_o, theta, decay)
    qe, ke = ltn.ltn_prologue_fwd(xqd, thd), ltn.ltn_prologue_fwd(xkd, thd)
    dqe, dke, dv = ltn.ltn_attn_bwd_dkdv(qe, ke, vd, gd, dd)
    dxq, dthq = ltn.ltn_prologue_bwd(xqd, dqe, thd)
    dxk, dthk = ltn.ltn_prologue_bwd(xkd, dke, thd)
    tol = TOL[dtype]
    check("dv", dv, dv_r, tol)
    check("dxq", dxq, dxq_r, tol)
    check("dxk", dxk, dxk_r, tol)
    assert orc.rel_l2(dthq + dthk, dthq_r + dthk_r) <= tol


def test_first_layer_chain_on_a_side_stream_and_in_a_graph():
    """The first-layer chain (expansion, attention, gradients, the expansion's derivative) is
    enqueued on the caller's stream and can be captured: replays with fresh inputs, with eager
    work in between, give the eager results bit for bit (no atomics, no memset nodes)."""
    Bt, H, N, D = 2, 4, 200, 128
    dtype = torch.bfloat16
    dd, th = gpu(synth.decay_bench_rule(H), synth.make_theta(H, D, 680))
    xq, xk, v, g = (torch.empty(Bt, H, N, D, dtype=dtype, device=dev()) for _ in range(4))

    def fill(seed):
        xq.copy_(synth.make_preact(Bt, H, N, D, dtype, seed, 0).to(dev()))
        xk.copy_(synth.make_preact(Bt, H, N, D, dtype, seed, 1).to(dev()))
        v.copy_(synth.make_qkv(Bt, H, N, D, dtype, seed)[2].to(dev()))
        g.copy_(synth.make_do(Bt, H, N, D, dtype, seed).to(dev()))

    def chain():
        qe, ke = ltn.ltn_prologue_fwd(xq, th, pos0=7), ltn.ltn_prologue_fwd(xk, th, pos0=7)
        o = ltn.ltn_attn_fwd_dkdv(qe, ke, v, dd)
        dqe, dke, dv = ltn.ltn_attn_bwd_dkdv(qe, ke, v, g, dd)
        dxq, dthq = ltn.ltn_prologue_bwd(xq, dqe, th, pos0=7)
        dxk, dthk = ltn.ltn_prologue_bwd(xk, dke, th, pos0=7)
        return [o, dv, dxq, dxk, dthq, dthk]

    fill(1)
    ref = chain()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        on_side = chain()
    side.synchronize()
    for a, b in zip(on_side, ref):
        assert torch.equal(a, b)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        outs = chain()
    for seed in (2, 3, 4):
        fill(seed)
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in outs]
        want = chain()                                   # eager, between replays
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b), seed
