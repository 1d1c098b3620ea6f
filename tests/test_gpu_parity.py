"""GPU parity: the HIP library (through its C ABI, via the ctypes binding) against the
fp64 CPU oracle, element by element on the same seeded inputs.

Error metric: ||x - ref||_2 / ||ref||_2 in fp64, maximum over the whole tensor and
every (batch, head) slice.  Bounds: 1e-4 for fp32 tensors, 1e-2 for bf16 tensors
(bf16 inputs are widened exactly for the oracle, so the bound covers the kernel's own
arithmetic: bf16 rounding of the masked scores, of the published state and of the
outputs, with fp32 accumulation).
"""
import numpy as np
import pytest
import torch

import paper_2307_14995_amd as ltn
from paper_2307_14995_amd import synth
from oracle import ltn_oracle as orc
from _helpers import TOL, TOL_ROW, check, check_rows, decays, dev, force_dv, force_plan, force_segs, gpu, mixed_decay

pytestmark = pytest.mark.gpu


# --------------------------------------------------------------------------- config 1 (fp32)


def test_cfg1_fp32_forward():
    w = synth.CONFIGS["cfg1_fp32_small"]
    q, k, v = synth.make_qkv(w.Bt, w.H, w.N, w.D, w.dtype, w.seed)
    decay = synth.decay_bench_rule(w.H)
    o = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), block=w.block)
    ref = orc.fwd_quadratic(q, k, v, decay)
    check("O", o, ref, 1e-4)


@pytest.mark.parametrize("D,block", [(64, 16), (64, 32), (64, 64), (128, 16), (128, 32)])
@pytest.mark.parametrize("N", [1, 37, 130])
def test_fp32_fwd_bwd_blocks(D, block, N):
    Bt, H = 2, 3
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.float32, 100 + N)
    g = synth.make_do(Bt, H, N, D, torch.float32, 100 + N)
    decay = decays(H)["mix"]
    for dv in (D, D // 2, D // 4):       # a split the kernels do not have for this block falls back to the library's choice
        with force_dv(dv):
            o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), block=block, return_state=True)
            dq, dk, dvv = ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay), block=block)
        o_ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, return_state=True)
        check("O", o, orc.fwd_quadratic(q, k, v, decay), 1e-4)
        check("kv", kv, kv_ref, 1e-4)
        for n, x, r in zip(("dQ", "dK", "dV"), (dq, dk, dvv), orc.bwd_quadratic(q, k, v, g, decay)):
            check(n, x, r, 1e-4)


def test_fp32_state_in_chunked_and_many_chains():
    """fp32 on the matrix cores: 16 chains (the XCD-grouped workgroup map), an initial state, a
    chunked prefill cut off a block boundary, ragged length."""
    Bt, H, N, D = 2, 8, 333, 128
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.float32, 111)
    g = synth.make_do(Bt, H, N, D, torch.float32, 111)
    kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(5)) * 0.1
    decay = decays(H)["mix"]
    qd, kd, vd, gd, dd, kv0d = gpu(q, k, v, g, decay, kv0)
    ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
    o, kv = ltn.ltn_attn_fwd(qd, kd, vd, dd, kv_in=kv0d, return_state=True)
    check("O", o, ref, 1e-4)
    check_rows("O rows", o, ref, TOL_ROW[torch.float32])
    check("kv", kv, kv_ref, 1e-4)
    cut = 77
    o1, kv1 = ltn.ltn_attn_fwd(qd[:, :, :cut].contiguous(), kd[:, :, :cut].contiguous(), vd[:, :, :cut].contiguous(),
                               dd, kv_in=kv0d, return_state=True)
    o2, kv2 = ltn.ltn_attn_fwd(qd[:, :, cut:].contiguous(), kd[:, :, cut:].contiguous(), vd[:, :, cut:].contiguous(),
                               dd, kv_in=kv1, return_state=True)
    check("O chunked", torch.cat([o1, o2], 2), ref, 1e-4)
    check("kv chunked", kv2, kv_ref, 1e-4)
    for n, x, r in zip(("dQ", "dK", "dV"), ltn.ltn_attn_bwd(qd, kd, vd, gd, dd), orc.bwd_recurrent(q, k, v, g, decay)):
        check(n, x, r, 1e-4)
        check_rows(n + " rows", x, r, TOL_ROW[torch.float32])


def test_cfg2_385m_shape_in_fp32_every_chain():
    """The 385M-shaped layer with fp32 tensors (the fp32 MFMA kernel at the shape its timing is
    quoted on): every chain, slice by slice and token by token."""
    w = synth.CONFIGS["cfg2_385m"]
    q, k, v = synth.make_qkv(w.Bt, w.H, w.N, w.D, torch.float32, w.seed)
    g = synth.make_do(w.Bt, w.H, w.N, w.D, torch.float32, w.seed)
    decay = synth.decay_bench_rule(w.H)
    qd, kd, vd, gd, dd = gpu(q, k, v, g, decay)
    o = ltn.ltn_attn_fwd(qd, kd, vd, dd).cpu()
    grads = tuple(x.cpu() for x in ltn.ltn_attn_bwd(qd, kd, vd, gd, dd))
    for b in range(w.Bt):
        sl = slice(b, b + 1)
        refs = (orc.fwd_recurrent(q[sl], k[sl], v[sl], decay),) + tuple(orc.bwd_recurrent(q[sl], k[sl], v[sl], g[sl], decay))
        for n, x, r in zip(("O", "dQ", "dK", "dV"), (o,) + grads, refs):
            check(f"{n}[{b}]", x[sl], r, 1e-4)
            check_rows(f"{n}[{b}] rows", x[sl], r, TOL_ROW[torch.float32])


# --------------------------------------------------------------------------- bf16 forward


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("N", [1, 15, 63, 64, 65, 128, 200, 517])
def test_bf16_forward_ragged(D, N):
    Bt, H = 1, 3                           # 3 chains: the non-XCD-grouped workgroup map
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 200 + N)
    for name, decay in decays(H).items():
        ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, return_state=True)
        for dv in (D, D // 2) + ((D // 4,) if D == 128 else ()):
            with force_dv(dv):
                o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), return_state=True)
            check(f"O[{name},dv={dv}]", o, ref, 1e-2)
            check(f"kv[{name},dv={dv}]", kv, kv_ref, 1e-2)


def test_bf16_forward_many_chains_xcd_map():
    Bt, H, N, D = 4, 8, 300, 128           # 32 chains: the XCD-grouped workgroup map
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 31)
    decay = synth.decay_bench_rule(H)
    ref = orc.fwd_recurrent(q, k, v, decay)
    for dv in (128, 64, 32):
        with force_dv(dv):
            o = ltn.ltn_attn_fwd(*gpu(q, k, v, decay))
        check(f"O[dv={dv}]", o, ref, 1e-2)


def test_bf16_chunked_prefill_matches_one_call():
    Bt, H, N, D = 2, 4, 448, 128
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 41)
    decay = decays(H)["mix"]
    qd, kd, vd, dd = gpu(q, k, v, decay)
    ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    cut = 203                               # not a block multiple
    o1, kv1 = ltn.ltn_attn_fwd(qd[:, :, :cut].contiguous(), kd[:, :, :cut].contiguous(),
                               vd[:, :, :cut].contiguous(), dd, return_state=True)
    o2, kv2 = ltn.ltn_attn_fwd(qd[:, :, cut:].contiguous(), kd[:, :, cut:].contiguous(),
                               vd[:, :, cut:].contiguous(), dd, kv_in=kv1, return_state=True)
    check("O", torch.cat([o1, o2], 2), ref, 1e-2)
    check("kv", kv2, kv_ref, 1e-2)
    # N = 0 with a state: the state is passed through untouched
    empty = qd[:, :, :0].contiguous()
    _, kv3 = ltn.ltn_attn_fwd(empty, empty, empty, dd, kv_in=kv2, return_state=True)
    assert torch.equal(kv3, kv2)
    _, kv4 = ltn.ltn_attn_fwd(empty, empty, empty, dd, return_state=True)
    assert torch.count_nonzero(kv4) == 0


# --------------------------------------------------------------------------- bf16 backward


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("N", [1, 64, 97, 333])
def test_bf16_backward_ragged(D, N):
    Bt, H = 2, 3
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 300 + N)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 300 + N)
    for name, decay in decays(H).items():
        refs = orc.bwd_recurrent(q, k, v, g, decay)
        for dv in (D, D // 2) + ((D // 4,) if D == 128 else ()):
            with force_dv(dv):
                outs = ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay))
            for n, x, r in zip(("dQ", "dK", "dV"), outs, refs):
                check(f"{n}[{name},dv={dv}]", x, r, 1e-2)


@pytest.mark.parametrize("chains,D", [(9, 128), (20, 128), (42, 128), (13, 64), (82, 96), (9, 256), (260, 64)])
def test_bf16_chain_counts_off_the_multiples_of_eight(chains, D):
    """Chain counts that are no multiple of 8: the launch is padded to whole groups of 8 chain
    slots while an XCD's share of workgroups fits its compute units (9 .. 42 chains here), else
    ids stay chain-major (82 chains of three slices, 260 chains); the empty slots' workgroups must
    touch nothing, every chain must be computed once, at every slice width."""
    Bt, H, N = 1, chains, 200
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 3100 + chains)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 3100 + chains)
    decay = mixed_decay(H)
    ref, ref_kv = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    refs = orc.bwd_recurrent(q, k, v, g, decay)
    widths = {64: (0, 32, 64), 96: (0, 32, 96), 128: (0, 32, 64, 128), 256: (0, 32, 64)}[D]
    for dv in widths:
        with force_plan(dv, 1 if dv else 0):
            o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), return_state=True)
            grads = ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay))
        check(f"o[dv={dv}]", o, ref, 1e-2)
        check(f"kv[dv={dv}]", kv, ref_kv, 1e-2)
        for n, x, r in zip(("dQ", "dK", "dV"), grads, refs):
            check(f"{n}[dv={dv}]", x, r, 1e-2)


def test_bf16_backward_probe_reads_back_scores():
    """dO = e_t e_j^T: column j of dV must be row t of the masked score matrix A."""
    Bt, H, N, D = 1, 1, 150, 128
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 51)
    decay = torch.tensor([0.97], dtype=torch.float32)
    t, j = 140, 77
    g = torch.zeros(Bt, H, N, D, dtype=torch.bfloat16)
    g[0, 0, t, j] = 1.0
    _, _, dv = ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay))
    lam = float(decay[0])                   # the fp32 value the kernel sees
    a_row = (q[0, 0, t].double() @ k[0, 0].double().T) * torch.tensor(
        [lam ** (t - s) if s <= t else 0.0 for s in range(N)], dtype=torch.float64)
    assert orc.rel_l2(dv[0, 0, :, j], a_row.numpy()) <= 1e-2
    other = dv[0, 0].clone()
    other[:, j] = 0
    assert torch.count_nonzero(other) == 0


# --------------------------------------------------------------------------- decode


@pytest.mark.parametrize("dtype,D", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 128), (torch.float32, 64)])
def test_decode_steps_continue_prefix(dtype, D):
    Bt, H, N0, steps = 3, 4, 100, 24
    q, k, v = synth.make_qkv(Bt, H, N0, D, dtype, 61)
    decay = decays(H)["mix"]
    qd, kd, vd, dd = gpu(q, k, v, decay)
    _, kv = ltn.ltn_attn_fwd(qd, kd, vd, dd, return_state=True)
    _, kv_ref = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    tol = TOL[dtype]
    for s in range(steps):
        q1, k1, v1 = synth.make_step_qkv(Bt, H, D, dtype, 61, s)
        o1 = ltn.ltn_attn_decode_step(*gpu(q1, k1, v1), kv, dd)
        o_ref, kv_ref = orc.decode_step(q1, k1, v1, kv_ref, decay)
        check(f"o[{s}]", o1, o_ref, tol, per_slice=False)
    check("kv", kv, kv_ref, tol)


@pytest.mark.parametrize("dtype,D", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 128), (torch.float32, 64)])
@pytest.mark.parametrize("S", [1, 5, 17])
def test_decode_several_tokens_per_call(dtype, D, S):
    """S iterations of Algorithm 2 in one call: rows of a forward that continues the state,
    and bit for bit what S single-token calls give."""
    Bt, H = 2, 5
    decay = decays(H)["mix"]
    g = torch.Generator().manual_seed(77 + S)
    kv0 = torch.randn(Bt, H, D, D, generator=g) * 0.2
    q, k, v = synth.make_qkv(Bt, H, S, D, dtype, 63 + S)
    dd, = gpu(decay)
    kv = kv0.to(dev())
    o = ltn.ltn_attn_decode_steps(*gpu(q, k, v), kv, dd)
    o_ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
    tol = TOL[dtype]
    check("o", o, o_ref, tol, per_slice=(S >= 5))
    check("kv", kv, kv_ref, tol)
    kv1 = kv0.to(dev())
    qd, kd, vd = gpu(q, k, v)
    for s_ in range(S):
        o1 = ltn.ltn_attn_decode_step(qd[:, :, s_].contiguous(), kd[:, :, s_].contiguous(),
                                      vd[:, :, s_].contiguous(), kv1, dd)
        assert torch.equal(o1, o[:, :, s_])
    assert torch.equal(kv1, kv)
    # S = 0: nothing happens
    empty = qd[:, :, :0].contiguous()
    assert ltn.ltn_attn_decode_steps(empty, empty, empty, kv1, dd).shape == (Bt, H, 0, D)
    assert torch.equal(kv1, kv)


# --------------------------------------------------------------------------- determinism / robustness


def test_bitwise_reproducible():
    Bt, H, N, D = 2, 4, 260, 128
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 71)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 71)
    args = gpu(q, k, v, g, synth.decay_bench_rule(H))
    a = ltn.ltn_attn_fwd(*args[:3], args[4])
    b = ltn.ltn_attn_fwd(*args[:3], args[4])
    assert torch.equal(a, b)
    ga = ltn.ltn_attn_bwd(*args)
    gb = ltn.ltn_attn_bwd(*args)
    for x, y in zip(ga, gb):
        assert torch.equal(x, y)


def test_outputs_fully_overwritten_and_inputs_untouched():
    Bt, H, N, D = 1, 2, 100, 128
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 81)
    decay = synth.decay_bench_rule(H)
    qd, kd, vd, dd = gpu(q, k, v, decay)
    poison = torch.full_like(qd, float("nan"))
    o = ltn.ltn_attn_fwd(qd, kd, vd, dd, out=poison)
    assert torch.isfinite(o.float()).all()
    assert torch.equal(qd.cpu(), q) and torch.equal(kd.cpu(), k) and torch.equal(vd.cpu(), v)


def test_strong_decay_stays_finite_on_long_sequence():
    """exp(-8) per token: the factorised form of Algorithm 1 would overflow; ours must not."""
    Bt, H, N, D = 1, 2, 2048, 128
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 91)
    decay = torch.tensor([float(np.exp(-8.0)), 1.0], dtype=torch.float32)
    o = ltn.ltn_attn_fwd(*gpu(q, k, v, decay))
    check("O", o, orc.fwd_recurrent(q, k, v, decay), 1e-2)


# --------------------------------------------------------------------------- full-size configurations


def every_chain_check(w):
    """Run the full-size workload on the GPU in the benchmark's launch configuration and
    compare EVERY (b,h) chain's O, dQ, dK, dV against the oracle (batch entry by batch entry,
    to bound host memory): the slice metric at the parity bound, and every token row at the
    per-token bound, so that a fault confined to a block, a segment seam or one workgroup's
    rows cannot hide inside a slice norm."""
    q, k, v = synth.make_qkv(w.Bt, w.H, w.N, w.D, w.dtype, w.seed)
    g = synth.make_do(w.Bt, w.H, w.N, w.D, w.dtype, w.seed)
    decay = synth.decay_bench_rule(w.H)
    qd, kd, vd, gd, dd = gpu(q, k, v, g, decay)
    o = ltn.ltn_attn_fwd(qd, kd, vd, dd, block=w.block)
    grads = ltn.ltn_attn_bwd(qd, kd, vd, gd, dd, block=w.block)
    torch.cuda.synchronize()
    o = o.cpu()
    grads = tuple(x.cpu() for x in grads)
    tol, tol_row = TOL[w.dtype], TOL_ROW[w.dtype]
    worst = {}
    for b in range(w.Bt):
        sl = slice(b, b + 1)
        refs = (orc.fwd_recurrent(q[sl], k[sl], v[sl], decay),) + tuple(orc.bwd_recurrent(q[sl], k[sl], v[sl], g[sl], decay))
        for n, x, r in zip(("O", "dQ", "dK", "dV"), (o,) + grads, refs):
            e = check(f"{n}[{b}]", x[sl], r, tol)
            er = check_rows(f"{n}[{b}] rows", x[sl], r, tol_row)
            worst[n] = max(worst.get(n, (0, 0)), (e, er))
    print(w.name, {n: f"slice {e:.2e} row {er:.2e}" for n, (e, er) in worst.items()})


def test_cfg2_385m_shape_every_chain():
    every_chain_check(synth.CONFIGS["cfg2_385m"])


def test_cfg_1b_shape_every_chain():
    every_chain_check(synth.CONFIGS["cfg_1b"])


def test_cfg3_7b_shape_every_chain():
    every_chain_check(synth.CONFIGS["cfg3_7b"])


def test_long_context_every_chain():
    """Bt=1, H=32, D=128, N=65536 (the launch configuration the report times): every chain against the
    oracle, slice by slice and token by token.  (Time against N: tests/test_gpu_timing.py.)"""
    H, D, N = 32, 128, 65536
    decay = synth.decay_bench_rule(H)
    q, k, v = synth.make_qkv(1, H, N, D, torch.bfloat16, synth.LONG_CONTEXT_SEED)
    g = synth.make_do(1, H, N, D, torch.bfloat16, synth.LONG_CONTEXT_SEED)
    qd, kd, vd, gd, dd = gpu(q, k, v, g, decay)
    oc = ltn.ltn_attn_fwd(qd, kd, vd, dd).cpu()
    gc = tuple(x.cpu() for x in ltn.ltn_attn_bwd(qd, kd, vd, gd, dd))
    refs = (orc.fwd_recurrent(q, k, v, decay),) + tuple(orc.bwd_recurrent(q, k, v, g, decay))
    for n, x, r in zip(("O", "dQ", "dK", "dV"), (oc,) + gc, refs):
        check(n, x, r, 1e-2)
        check_rows(n + " rows", x, r, TOL_ROW[torch.bfloat16])


def test_decode_config5_all_steps_all_chains():
    """Bt=64, H=32, D=128: state from a 1024-token prefix (every chain's state against the
    oracle), then all 512 decode steps.  Every step's output [Bt,H,D] is compared for sampled
    chains step by step (the oracle's decode_step), and for EVERY chain through one oracle
    forward over the 512 step tokens that continues the prefix state (Algorithm 2 is the same
    loop either way); the final state of every chain is compared too."""
    c = synth.DECODE
    Bt, H, D, N0, steps = c["Bt"], c["H"], c["D"], c["prefix"], c["steps"]
    q, k, v = synth.make_qkv(Bt, H, N0, D, torch.bfloat16, c["seed"])
    decay = synth.decay_bench_rule(H)
    qd, kd, vd, dd = gpu(q, k, v, decay)
    _, kv = ltn.ltn_attn_fwd(qd, kd, vd, dd, return_state=True)
    _, kv0_ref = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    check("kv0", kv, kv0_ref, 1e-2)
    picks = [(0, 0), (17, 9), (63, 31)]
    ref_state = {bh: kv0_ref[bh[0]:bh[0] + 1, bh[1]:bh[1] + 1] for bh in picks}
    qs, ks, vs = (torch.empty(Bt, H, steps, D, dtype=torch.bfloat16) for _ in range(3))
    outs = torch.empty(Bt, H, steps, D, dtype=torch.bfloat16)
    for s in range(steps):
        q1, k1, v1 = synth.make_step_qkv(Bt, H, D, torch.bfloat16, c["seed"], s)
        qs[:, :, s], ks[:, :, s], vs[:, :, s] = q1, k1, v1
        o1 = ltn.ltn_attn_decode_step(*gpu(q1, k1, v1), kv, dd)
        outs[:, :, s] = o1.cpu()
        for (b, h) in picks:
            sl = (slice(b, b + 1), slice(h, h + 1))
            o_ref, ref_state[(b, h)] = orc.decode_step(q1[sl], k1[sl], v1[sl], ref_state[(b, h)], decay[h:h + 1])
            check(f"o[{s}][{b},{h}]", o1[sl], o_ref, 1e-2)
    kv = kv.cpu()
    for (b, h) in picks:
        sl = (slice(b, b + 1), slice(h, h + 1))
        check(f"kv[{b},{h}]", kv[sl], ref_state[(b, h)], 1e-2)
    # every chain: the 512 step tokens as one Algorithm-2 run from the prefix state
    o_all, kv_ref = orc.fwd_recurrent(qs, ks, vs, decay, kv_in=kv0_ref, return_state=True)
    check("o (all steps, all chains)", outs, o_all, 1e-2)
    check_rows("o rows", outs, o_all, TOL_ROW[torch.bfloat16])
    check("kv (all chains)", kv, kv_ref, 1e-2)


# --------------------------------------------------------------------------- sequence-parallel form


@pytest.mark.parametrize("D", [64, 96, 128, 256])
@pytest.mark.parametrize("N,segs", [(130, 2), (517, 3), (1000, 5), (640, 10)])
def test_bf16_segmented_forward_backward(D, N, segs):
    """Chains cut into segments (end states from zero, scan, per-segment pass) give the same
    O, final state and gradients as the definition; initial state included."""
    Bt, H = 1, 3
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 600 + N)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 600 + N)
    kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(N)) * 0.1
    decay = decays(H)["mix"]
    ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
    refs = orc.bwd_recurrent(q, k, v, g, decay)
    with force_segs(segs):
        assert ltn.ltn_attn_workspace_bytes(Bt, H, N, D, 0, torch.bfloat16, 0) > 0
        o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), kv_in=kv0.to(dev()), return_state=True)
        o2 = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), kv_in=kv0.to(dev()))      # final state not requested
        outs = ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay))
    check("O", o, ref, 1e-2)
    check("kv", kv, kv_ref, 1e-2)
    assert torch.equal(o2, o)
    for n, x, r in zip(("dQ", "dK", "dV"), outs, refs):
        check(n, x, r, 1e-2)


def test_bf16_segmented_by_default_for_few_long_chains():
    Bt, H, N, D = 1, 2, 8192 + 77, 128
    assert ltn.ltn_attn_workspace_bytes(Bt, H, N, D, 0, torch.bfloat16, 0) > 0
    assert ltn.ltn_attn_workspace_bytes(Bt, H, N, D, 0, torch.bfloat16, 1) > 0
    assert ltn.ltn_attn_workspace_bytes(4, 32, 8192, D, 0, torch.bfloat16, 1) == 0    # headline shape: whole chains
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 91)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 91)
    decay = synth.decay_bench_rule(H)
    o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), return_state=True)
    ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    check("O", o, ref, 1e-2)
    check("kv", kv, kv_ref, 1e-2)
    for n, x, r in zip(("dQ", "dK", "dV"), ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay)),
                       orc.bwd_recurrent(q, k, v, g, decay)):
        check(n, x, r, 1e-2)


def test_one_very_long_chain():
    """A single chain of 262144 tokens: the deepest cut the library's rule makes (256 segments, one
    per compute unit), forward with the final state and backward, every token row against the oracle."""
    Bt, H, N, D = 1, 1, 262144, 64
    assert ltn.ltn_attn_query_plan(Bt, H, N, D, torch.bfloat16, 0)[1] == 256
    # backward: 85 ways at most for three passes, cut to 72 so that chains x segments is a multiple of 8
    assert ltn.ltn_attn_workspace_bytes(Bt, H, N, D, 0, torch.bfloat16, 1) == 3 * 72 * D * D * 4
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 97)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 97)
    decay = torch.tensor([float(np.exp(-1.0 / 512.0))])
    o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), return_state=True)
    grads = ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay))
    ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    refs = orc.bwd_recurrent(q, k, v, g, decay)
    check("O", o, ref, 1e-2)
    check_rows("O rows", o, ref, TOL_ROW[torch.bfloat16])
    check("kv", kv, kv_ref, 1e-2)
    for n, x, r in zip(("dQ", "dK", "dV"), grads, refs):
        check(n, x, r, 1e-2)
        check_rows(n + " rows", x, r, TOL_ROW[torch.bfloat16])


def test_segmented_call_needs_its_workspace():
    Bt, H, N, D = 1, 2, 8192, 128
    q, k, v = gpu(*synth.make_qkv(Bt, H, N, D, torch.bfloat16, 93))
    dd, = gpu(synth.decay_bench_rule(H))
    o = torch.empty_like(q)
    lib = ltn.load_library()
    import ctypes
    need = ltn.ltn_attn_workspace_bytes(Bt, H, N, D, 0, torch.bfloat16, 0)
    assert need == 16 * Bt * H * D * D * 4              # 8192 tokens: sixteen segments of 512
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = lib.ltn_attn_fwd(p(q), p(k), p(v), p(o), p(dd), None, None, Bt, H, N, D, 0, 1, None, 0, None)
    assert rc == 2, ltn.ltn_status_str(rc)               # LTN_ERR_SHAPE: workspace too small
    rc = lib.ltn_attn_fwd(p(q), p(k), p(v), p(o), p(dd), None, None, Bt, H, N, D, 0, 1, None, need, None)
    assert rc == 1, ltn.ltn_status_str(rc)               # LTN_ERR_NULL: bytes needed, no pointer


# --------------------------------------------------------------------------- seeded sweep of odd shapes


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        Bt, H = int(rng.integers(1, 4)), int(rng.integers(1, 10))
        N = int(rng.choice([rng.integers(1, 64), rng.integers(64, 400), rng.integers(400, 1500)]))
        dv = int(rng.choice([D, D // 2] + ([D // 4] if D == 128 else [])))
        segs = int(rng.choice([1, 1, 2, 3, 7]))
        cases.append((i, Bt, H, N, D, dv, segs))
    return cases


@pytest.mark.parametrize("case", _random_cases(16, 2024), ids=lambda c: "B%dH%dN%dD%ddv%dseg%d" % c[1:])
def test_bf16_seeded_shape_sweep(case):
    """Forward (with an initial state, returning the final one) and backward on seeded odd
    shapes, value-column split and segment count forced, against the oracle."""
    i, Bt, H, N, D, dv, segs = case
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 700 + i)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 700 + i)
    kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(i)) * 0.1
    decay = torch.rand(H, generator=torch.Generator().manual_seed(1000 + i))
    decay[0] = 1.0
    ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
    refs = orc.bwd_recurrent(q, k, v, g, decay)
    with force_plan(dv, segs):
        o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), kv_in=kv0.to(dev()), return_state=True)
        outs = ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay))
    check("O", o, ref, 1e-2)
    check("kv", kv, kv_ref, 1e-2)
    for n, x, r in zip(("dQ", "dK", "dV"), outs, refs):
        check(n, x, r, 1e-2)


def _random_cases_f32(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        Bt, H = int(rng.integers(1, 4)), int(rng.integers(1, 10))
        N = int(rng.choice([rng.integers(1, 64), rng.integers(64, 400), rng.integers(400, 900)]))
        block = int(rng.choice([0, 16, 32] + ([64] if D == 64 else [])))
        dv = int(rng.choice([0, D, D // 2, D // 4]))      # widths a kernel lacks are ignored by the library
        cases.append((i, Bt, H, N, D, block, dv))
    return cases


@pytest.mark.parametrize("case", _random_cases_f32(12, 2025), ids=lambda c: "B%dH%dN%dD%dblk%ddv%d" % c[1:])
def test_fp32_seeded_shape_sweep(case):
    """fp32 tensors: forward (initial state in, final state out) and backward on seeded odd
    shapes, block length and value-column split forced, against the oracle."""
    i, Bt, H, N, D, block, dv = case
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.float32, 900 + i)
    g = synth.make_do(Bt, H, N, D, torch.float32, 900 + i)
    kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(50 + i)) * 0.1
    decay = torch.rand(H, generator=torch.Generator().manual_seed(1100 + i))
    decay[-1] = 0.0
    ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
    refs = orc.bwd_recurrent(q, k, v, g, decay)
    with force_plan(dv, 0):
        o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), kv_in=kv0.to(dev()), return_state=True, block=block)
        outs = ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay), block=block)
    check("O", o, ref, 1e-4)
    check("kv", kv, kv_ref, 1e-4)
    check_rows("O rows", o, ref, TOL_ROW[torch.float32])
    for n, x, r in zip(("dQ", "dK", "dV"), outs, refs):
        check(n, x, r, 1e-4)
        check_rows(n + " rows", x, r, TOL_ROW[torch.float32])


def _random_cases_wide(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        D = int(rng.choice([96, 256]))
        Bt, H = int(rng.integers(1, 3)), int(rng.integers(1, 7))
        N = int(rng.choice([rng.integers(1, 64), rng.integers(64, 400), rng.integers(400, 1200)]))
        segs = int(rng.choice([1, 1, 2, 3, 5]))
        dv = int(rng.choice([0, 32, 64] if D == 256 else [0, 32, 96, 96]))
        cases.append((i, Bt, H, N, D, dv, segs))
    return cases


@pytest.mark.parametrize("case", _random_cases_wide(10, 2026), ids=lambda c: "B%dH%dN%dD%ddv%dseg%d" % c[1:])
def test_bf16_wide_heads_seeded_shape_sweep(case):
    """Heads of 96 and 256 features on seeded odd shapes, segment count forced."""
    i, Bt, H, N, D, dv, segs = case
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 950 + i)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 950 + i)
    kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(70 + i)) * 0.1
    decay = torch.rand(H, generator=torch.Generator().manual_seed(1200 + i))
    decay[0] = 1.0
    ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
    refs = orc.bwd_recurrent(q, k, v, g, decay)
    with force_plan(dv, segs):
        o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), kv_in=kv0.to(dev()), return_state=True)
        outs = ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay))
    check("O", o, ref, 1e-2)
    check("kv", kv, kv_ref, 1e-2)
    for n, x, r in zip(("dQ", "dK", "dV"), outs, refs):
        check(n, x, r, 1e-2)


# --------------------------------------------------------------------------- the paper's tiling as a kernel


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("N", [1, 63, 64, 65, 200, 517])
def test_bf16_tiled_forward(D, N):
    """App. B Algorithm 3 evaluated on the GPU: the definition's O, by the quadratic tile loop."""
    Bt, H = 1, 3
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 800 + N)
    for name, decay in decays(H).items():
        o = ltn.ltn_attn_fwd_tiled(*gpu(q, k, v, decay))
        check(f"O[{name}]", o, orc.fwd_quadratic(q, k, v, decay), 1e-2)
    # the oracle's own Algorithm 3 (64 x 64 tiles) is the same numbers
    assert orc.rel_l2(orc.fwd_tiled(q, k, v, decays(H)["bench"], 64, 64),
                      orc.fwd_quadratic(q, k, v, decays(H)["bench"])) < 1e-12


def test_bf16_tiled_forward_many_chains_long():
    Bt, H, N, D = 2, 8, 1500, 128           # 16 chains (XCD-grouped), 24 query blocks each
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 87)
    decay = synth.decay_bench_rule(H)
    o = ltn.ltn_attn_fwd_tiled(*gpu(q, k, v, decay))
    check("O", o, orc.fwd_recurrent(q, k, v, decay), 1e-2)
    with pytest.raises(ltn.LtnError):
        ltn.ltn_attn_fwd_tiled(*gpu(q.float(), k.float(), v.float(), decay))     # bf16 only


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("N", [1, 63, 64, 65, 200, 517])
def test_bf16_tiled_backward(D, N):
    """App. B Algorithm 4 (corrected) evaluated on the GPU: the gradients of the definition, by
    the quadratic tile loops (one workgroup per key/value block for dK, dV; one per query block
    for dQ)."""
    Bt, H = 1, 3
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 820 + N)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 820 + N)
    for name, decay in decays(H).items():
        outs = ltn.ltn_attn_bwd_tiled(*gpu(q, k, v, g, decay))
        for n, x, r in zip(("dQ", "dK", "dV"), outs, orc.bwd_quadratic(q, k, v, g, decay)):
            check(f"{n}[{name}]", x, r, 1e-2)


def test_bf16_tiled_backward_many_chains_long():
    Bt, H, N, D = 2, 8, 1500, 128           # 16 chains (XCD-grouped), 24 blocks each, ragged tail
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 89)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 89)
    decay = synth.decay_bench_rule(H)
    poison = tuple(torch.full((Bt, H, N, D), float("nan"), dtype=torch.bfloat16, device=dev()) for _ in range(3))
    outs = ltn.ltn_attn_bwd_tiled(*gpu(q, k, v, g, decay), out=poison)
    refs = orc.bwd_recurrent(q, k, v, g, decay)
    for n, x, r in zip(("dQ", "dK", "dV"), outs, refs):
        check(n, x, r, 1e-2)
        check_rows(n + " rows", x, r, TOL_ROW[torch.bfloat16])
    again = ltn.ltn_attn_bwd_tiled(*gpu(q, k, v, g, decay))
    for a, b in zip(outs, again):
        assert torch.equal(a, b)             # no atomics: reproducible bit for bit
    with pytest.raises(ltn.LtnError):
        ltn.ltn_attn_bwd_tiled(*gpu(q.float(), k.float(), v.float(), g.float(), decay))     # bf16 only


# --------------------------------------------------------------------------- cost linear in N


def test_work_goes_to_the_callers_stream():
    """The library enqueues on the stream it is handed (here torch's current stream) and does
    not synchronise: results on a side stream match the default-stream results bit for bit."""
    Bt, H, N, D = 2, 4, 300, 128
    q, k, v = gpu(*synth.make_qkv(Bt, H, N, D, torch.bfloat16, 97))
    g, = gpu(synth.make_do(Bt, H, N, D, torch.bfloat16, 97))
    dd, = gpu(synth.decay_bench_rule(H))
    o_ref = ltn.ltn_attn_fwd(q, k, v, dd)
    g_ref = ltn.ltn_attn_bwd(q, k, v, g, dd)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        o = ltn.ltn_attn_fwd(q, k, v, dd)
        grads = ltn.ltn_attn_bwd(q, k, v, g, dd)
    side.synchronize()
    assert torch.equal(o, o_ref)
    for a, b in zip(grads, g_ref):
        assert torch.equal(a, b)


def test_calls_can_be_captured_in_a_graph():
    """Forward + backward captured once and replayed: every replay, with eager work and fresh
    inputs in between, gives the eager results bit for bit (the calls allocate nothing and
    record no memset)."""
    Bt, H, N, D = 2, 4, 200, 128
    dd, = gpu(synth.decay_bench_rule(H))
    q, k, v, g = (torch.empty(Bt, H, N, D, dtype=torch.bfloat16, device=dev()) for _ in range(4))
    o = torch.empty_like(q)
    grads = tuple(torch.empty_like(q) for _ in range(3))

    def fill(seed):
        a, b, c = synth.make_qkv(Bt, H, N, D, torch.bfloat16, seed)
        q.copy_(a.to(dev())); k.copy_(b.to(dev())); v.copy_(c.to(dev()))
        g.copy_(synth.make_do(Bt, H, N, D, torch.bfloat16, seed).to(dev()))

    fill(1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside capture
        ltn.ltn_attn_fwd(q, k, v, dd, out=o)
        ltn.ltn_attn_bwd(q, k, v, g, dd, out=grads)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ltn.ltn_attn_fwd(q, k, v, dd, out=o)
        ltn.ltn_attn_bwd(q, k, v, g, dd, out=grads)
    for seed in (2, 3, 4):
        fill(seed)
        o.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [o.clone()] + [x.clone() for x in grads]
        want = [ltn.ltn_attn_fwd(q, k, v, dd)] + list(ltn.ltn_attn_bwd(q, k, v, g, dd))   # eager, between replays
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b), seed
