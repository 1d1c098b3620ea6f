"""GPU parity for heads of 256 features (forward, state hand-over, gradients, decode), through
the C ABI against the fp64 oracle; the same checks as for D = 64 and 128 at sizes the oracle
finishes quickly."""
import numpy as np
import pytest
import torch

import paper_2307_14995_amd as ltn
from paper_2307_14995_amd import synth
from oracle import ltn_oracle as orc
from _helpers import check, dev, gpu, mixed_decay

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-4, torch.bfloat16: 1e-2}
D = 256


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("N", [1, 63, 64, 65, 200, 517])
def test_d256_forward_ragged(dtype, N):
    Bt, H = 1, 3
    q, k, v = synth.make_qkv(Bt, H, N, D, dtype, 700 + N)
    decay = mixed_decay(H)
    o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), return_state=True)
    ref, ref_kv = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    check("o", o, ref, TOL[dtype])
    check("kv_out", kv, ref_kv, TOL[dtype])


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_d256_state_in_and_chunked_prefill(dtype):
    Bt, H, N, cut = 2, 2, 330, 130
    q, k, v = synth.make_qkv(Bt, H, N, D, dtype, 720)
    decay = synth.decay_bench_rule(H)
    kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(721))
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
def test_d256_backward(dtype, Bt, H, N):
    # 3 chains take 32-column slices in bf16, 96 chains 64-column slices
    q, k, v = synth.make_qkv(Bt, H, N, D, dtype, 740 + N)
    d_o = synth.make_do(Bt, H, N, D, dtype, 740 + N)
    decay = mixed_decay(H)
    qd, kd, vd, gd, dd = gpu(q, k, v, d_o, decay)
    check("o", ltn.ltn_attn_fwd(qd, kd, vd, dd), orc.fwd_recurrent(q, k, v, decay), TOL[dtype])
    for name, got, ref in zip(("dq", "dk", "dv"), ltn.ltn_attn_bwd(qd, kd, vd, gd, dd),
                              orc.bwd_recurrent(q, k, v, d_o, decay)):
        check(name, got, ref, TOL[dtype])


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_d256_decode_continues_a_prefix(dtype):
    Bt, H, N0, S = 2, 3, 100, 6
    q, k, v = synth.make_qkv(Bt, H, N0 + S, D, dtype, 760)
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


def test_d256_unsupported_variants():
    H = 2
    decay = synth.decay_bench_rule(H).to(dev())
    a = torch.zeros(1, H, 64, D, dtype=torch.bfloat16, device=dev())
    with pytest.raises(ltn.LtnError):
        ltn.ltn_attn_fwd_gated(a, a.clone(), a.clone(), a.clone(), decay, store_o=False)   # only with O stored
    with pytest.raises(ltn.LtnError):
        ltn.ltn_attn_fwd_tiled(a, a.clone(), a.clone(), decay)


def test_d256_segmented_by_default_for_few_long_chains():
    Bt, H, N = 1, 2, 8192 + 77
    need = ltn.ltn_attn_workspace_bytes(Bt, H, N, D, 0, torch.bfloat16, 0)
    assert need == 15 * Bt * H * D * D * 4              # fifteen segments of 576 tokens
    assert ltn.ltn_attn_workspace_bytes(4, 16, 8192, D, 0, torch.bfloat16, 0) == 0    # enough chains: whole chains
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 780)
    g = synth.make_do(Bt, H, N, D, torch.bfloat16, 780)
    decay = synth.decay_bench_rule(H)
    o, kv = ltn.ltn_attn_fwd(*gpu(q, k, v, decay), return_state=True)
    ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, return_state=True)
    check("O", o, ref, 1e-2)
    check("kv", kv, kv_ref, 1e-2)
    for n, x, r in zip(("dQ", "dK", "dV"), ltn.ltn_attn_bwd(*gpu(q, k, v, g, decay)),
                       orc.bwd_recurrent(q, k, v, g, decay)):
        check(n, x, r, 1e-2)
