"""GPU parity for heads of 96 features (computed on chip as 128 with zero columns) (forward, state hand-over, gradients, decode), through
the C ABI against the fp64 oracle; the same checks as for D = 64 and 128 at sizes the oracle
finishes quickly."""
import numpy as np
import pytest
import torch

import paper_2307_14995_amd as ltn
from paper_2307_14995_amd import synth
from oracle import ltn_oracle as orc
from _helpers import check, dev, force_plan, gpu, mixed_decay

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-4, torch.bfloat16: 1e-2}
D = 96


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("N", [1, 63, 64, 65, 200, 517])
def test_d96_forward_ragged(dtype, N):
    Bt, H = 1, 3
    q, k, v = synth.make_qkv(Bt, H, N, D, dtype, 800 + N)
    decay = mixed_decay(H)
    o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), return_state=True)
    ref, ref_kv = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    check("o", o, ref, TOL[dtype])
    check("kv_out", kv, ref_kv, TOL[dtype])


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_d96_state_in_and_chunked_prefill(dtype):
    Bt, H, N, cut = 2, 2, 330, 130
    q, k, v = synth.make_qkv(Bt, H, N, D, dtype, 820)
    decay = synth.decay_bench_rule(H)
    kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(821))
    ref, ref_kv = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
    qd, kd, vd, dd, kv0d = gpu(q, k, v, decay, kv0)
    o1, s1 = ltn.ltn_attn_fwd(qd[:, :, :cut].contiguous(), kd[:, :, :cut].contiguous(),
                              vd[:, :, :cut].contiguous(), dd, kv_in=kv0d, return_state=True)
    o2, s2 = ltn.ltn_attn_fwd(qd[:, :, cut:].contiguous(), kd[:, :, cut:].contiguous(),
                              vd[:, :, cut:].contiguous(), dd, kv_in=s1, return_state=True)
    check("chunked o", torch.cat([o1, o2], dim=2), ref, TOL[dtype])
    check("chunked kv", s2, ref_kv, TOL[dtype])


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("Bt,H,N", [(1, 3, 1), (1, 3, 65), (1, 3, 300), (4, 24, 130)])
def test_d96_backward(dtype, Bt, H, N):
    # three 32-column slices per chain whatever the number of chains
    q, k, v = synth.make_qkv(Bt, H, N, D, dtype, 840 + N)
    d_o = synth.make_do(Bt, H, N, D, dtype, 840 + N)
    decay = mixed_decay(H)
    qd, kd, vd, gd, dd = gpu(q, k, v, d_o, decay)
    check("o", ltn.ltn_attn_fwd(qd, kd, vd, dd), orc.fwd_recurrent(q, k, v, decay), TOL[dtype])
    for name, got, ref in zip(("dq", "dk", "dv"), ltn.ltn_attn_bwd(qd, kd, vd, gd, dd),
                              orc.bwd_recurrent(q, k, v, d_o, decay)):
        check(name, got, ref, TOL[dtype])


@pytest.mark.parametrize("dv", [32, 96])
@pytest.mark.parametrize("N", [1, 63, 65, 200, 517])
def test_d96_both_slice_widths(dv, N):
    """Three 32-column workgroups per chain, or one with all 96 columns (forced): forward with an
    initial state and the final state, and all three gradients."""
    Bt, H = 2, 3
    dtype = torch.bfloat16
    q, k, v = synth.make_qkv(Bt, H, N, D, dtype, 870 + N)
    d_o = synth.make_do(Bt, H, N, D, dtype, 870 + N)
    kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(N)) * 0.1
    decay = mixed_decay(H)
    ref, ref_kv = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
    refs = orc.bwd_recurrent(q, k, v, d_o, decay)
    with force_plan(dv=dv):
        assert ltn.ltn_attn_query_plan(Bt, H, N, D, dtype, 0)[0] == dv
        o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), kv_in=kv0.to(dev()), return_state=True)
        grads = ltn.ltn_attn_bwd(*gpu(q, k, v, d_o, decay))
    check("o", o, ref, TOL[dtype])
    check("kv_out", kv, ref_kv, TOL[dtype])
    for name, got, r in zip(("dq", "dk", "dv"), grads, refs):
        check(name, got, r, TOL[dtype])


def test_d96_many_chains_take_all_columns_in_one_workgroup():
    # 4 x 24 chains: the backward's 288 passes are more than one round of compute units even at full
    # width, the forward's 96 chains x 3 slices are not
    assert ltn.ltn_attn_query_plan(4, 24, 130, D, torch.bfloat16, 0) == (96, 1)
    assert ltn.ltn_attn_query_plan(4, 24, 130, D, torch.bfloat16, 1) == (96, 1)
    assert ltn.ltn_attn_query_plan(2, 24, 130, D, torch.bfloat16, 0) == (32, 1)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_d96_decode_continues_a_prefix(dtype):
    Bt, H, N0, S = 2, 3, 100, 6
    q, k, v = synth.make_qkv(Bt, H, N0 + S, D, dtype, 860)
    decay = mixed_decay(H)
    ref, ref_kv = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    qd, kd, vd, dd = gpu(q, k, v, decay)
    _, kv = ltn.ltn_attn_fwd(qd[:, :, :N0].contiguous(), kd[:, :, :N0].contiguous(),
                             vd[:, :, :N0].contiguous(), dd, return_state=True)
    o_a = ltn.ltn_attn_decode_steps(qd[:, :, N0:N0 + 4].contiguous(), kd[:, :, N0:N0 + 4].contiguous(),
                                    vd[:, :, N0:N0 + 4].contiguous(), kv, dd)
    outs = [o_a]
    for t in range(N0 + 4, N0 + S):
        outs.append(ltn.ltn_attn_decode_step(qd[:, :, t].contiguous(), kd[:, :, t].contiguous(),
                                             vd[:, :, t].contiguous(), kv, dd).unsqueeze(2))
    check("decode o", torch.cat(outs, dim=2), ref[:, :, N0:], TOL[dtype])
    check("decode kv", kv, ref_kv, TOL[dtype])


def test_d96_few_long_chains_are_cut_into_segments_by_default():
    Bt, H, N = 1, 4, 4096 + 33                  # 4 chains x 3 slices: cut 8 ways by the library's own rule
    assert ltn.ltn_attn_query_plan(Bt, H, N, D, torch.bfloat16, 0) == (32, 8)
    assert ltn.ltn_attn_workspace_bytes(Bt, H, N, D, 0, torch.bfloat16, 0) == 8 * Bt * H * D * D * 4
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 880)
    kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(881)) * 0.1
    decay = synth.decay_bench_rule(H)
    o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), kv_in=kv0.to(dev()), return_state=True)
    ref, ref_kv = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
    check("o", o, ref, 1e-2)
    check("kv", kv, ref_kv, 1e-2)


def test_d96_segments_of_whole_row_workgroups_by_default():
    """From 12 chain passes on the library cuts for its 96-column workgroups (one per chain, pass
    and segment): forward of 32 chains, backward of 8 (24 passes: 10 segments, 80 = a multiple of 8
    chain segments), with a ragged tail and a state handed in."""
    Bt, H, N = 1, 32, 4096 + 33
    assert ltn.ltn_attn_query_plan(Bt, H, N, D, torch.bfloat16, 0) == (96, 8)
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 884)
    kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(885)) * 0.1
    decay = mixed_decay(H)
    o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), kv_in=kv0.to(dev()), return_state=True)
    ref, ref_kv = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
    check("o", o, ref, 1e-2)
    check("kv", kv, ref_kv, 1e-2)
    Bt, H, N = 1, 8, 8192 + 70
    assert ltn.ltn_attn_query_plan(Bt, H, N, D, torch.bfloat16, 1) == (96, 10)
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 886)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 886)
    decay = mixed_decay(H)
    grads = ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay))
    refs = orc.bwd_recurrent(q, k, v, g, decay)
    for n, x, r in zip(("dq", "dk", "dv"), grads, refs):
        check(n, x, r, 1e-2)


def test_d96_unsupported_variants():
    H = 2
    decay = synth.decay_bench_rule(H).to(dev())
    a = torch.zeros(1, H, 64, D, dtype=torch.bfloat16, device=dev())
    with pytest.raises(ltn.LtnError):
        ltn.ltn_attn_fwd_gated(a.float(), a.float(), a.float(), a.float(), decay, store_o=False)   # fp32: only with O stored
    with pytest.raises(ltn.LtnError):
        ltn.ltn_attn_fwd_tiled(a, a.clone(), a.clone(), decay)
