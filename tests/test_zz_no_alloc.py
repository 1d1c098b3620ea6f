"""The forward entry point that uses the library's static scratch (ltn_attn_fwd_static), called
through the C ABI with raw ctypes: two calls in a row, the second on a smaller input, each
against ltn_attn_fwd with a caller workspace (same plan, same kernels: bit for bit) and
against the fp64 oracle at the parity bound.  No allocation happens between the two calls."""
import ctypes

import pytest
import torch

import paper_2307_14995_amd as ltn
from paper_2307_14995_amd import synth
from oracle import ltn_oracle as orc
from _helpers import check, dev, gpu

pytestmark = pytest.mark.gpu


def _p(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def test_static_scratch_forward_two_calls_in_a_row():
    lib = ltn.load_library()
    D, BF16 = 128, 1
    shapes = [(1, 4, 16384 + 40), (1, 2, 8192 + 77)]          # both cut into segments by the library's own rule
    # everything either call needs is allocated up front
    bufs = []
    for (Bt, H, N) in shapes:
        q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 1200 + H)
        decay = synth.decay_bench_rule(H)
        kv0 = torch.randn(Bt, H, D, D, generator=torch.Generator().manual_seed(H)) * 0.1
        need = ltn.ltn_attn_workspace_bytes(Bt, H, N, D, 0, torch.bfloat16, 0)
        assert 0 < need <= 16 << 20
        d = dict(shape=(Bt, H, N), cpu=(q, k, v, decay, kv0), dev=gpu(q, k, v, decay, kv0),
                 o_s=torch.full((Bt, H, N, D), float("nan"), dtype=torch.bfloat16, device=dev()),
                 o_w=torch.empty(Bt, H, N, D, dtype=torch.bfloat16, device=dev()),
                 kv_s=torch.empty(Bt, H, D, D, device=dev()), kv_w=torch.empty(Bt, H, D, D, device=dev()),
                 ws=torch.empty(need, dtype=torch.uint8, device=dev()), need=need)
        bufs.append(d)
    torch.cuda.synchronize()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # the two static-scratch calls back to back, nothing else in between
    for d in bufs:
        Bt, H, N = d["shape"]
        qd, kd, vd, dd, kv0d = d["dev"]
        rc = lib.ltn_attn_fwd_static(_p(qd), _p(kd), _p(vd), _p(d["o_s"]), _p(dd), _p(kv0d), _p(d["kv_s"]),
                                     Bt, H, N, D, 0, BF16, stream)
        assert rc == 0, ltn.ltn_status_str(rc)
    torch.cuda.synchronize()
    for d in bufs:
        Bt, H, N = d["shape"]
        qd, kd, vd, dd, kv0d = d["dev"]
        rc = lib.ltn_attn_fwd(_p(qd), _p(kd), _p(vd), _p(d["o_w"]), _p(dd), _p(kv0d), _p(d["kv_w"]),
                              Bt, H, N, D, 0, BF16, _p(d["ws"]), d["need"], stream)
        assert rc == 0, ltn.ltn_status_str(rc)
        torch.cuda.synchronize()
        assert torch.equal(d["o_s"], d["o_w"]) and torch.equal(d["kv_s"], d["kv_w"])
        q, k, v, decay, kv0 = d["cpu"]
        ref, kv_ref = orc.fwd_recurrent(q, k, v, decay, kv_in=kv0, return_state=True)
        check("O", d["o_s"], ref, 1e-2)
        check("kv", d["kv_s"], kv_ref, 1e-2)


def test_static_scratch_refuses_what_does_not_fit_and_needs_no_scratch_for_whole_chains():
    lib = ltn.load_library()
    D, BF16 = 128, 1
    Bt, H, N = 2, 3, 300
    q, k, v = synth.make_qkv(Bt, H, N, D, torch.bfloat16, 1210)
    decay = synth.decay_bench_rule(H)
    qd, kd, vd, dd = gpu(q, k, v, decay)
    o = torch.empty_like(qd)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = lib.ltn_attn_fwd_static(_p(qd), _p(kd), _p(vd), _p(o), _p(dd), None, None, Bt, H, N, D, 0, BF16, stream)
    assert rc == 0, ltn.ltn_status_str(rc)                     # whole chains: the scratch is not touched
    torch.cuda.synchronize()
    check("O", o, orc.fwd_recurrent(q, k, v, decay), 1e-2)
    try:                                                       # a forced plan beyond the static buffer
        ltn.ltn_attn_set_debug_plan(0, 4)
        Bt2, H2 = 8, 12                                        # 96 chains x 3 segments of 128 tokens x 64 KB = 18 MiB
        assert ltn.ltn_attn_workspace_bytes(Bt2, H2, N, D, 0, torch.bfloat16, 0) > 16 << 20
        rc = lib.ltn_attn_fwd_static(_p(qd), _p(kd), _p(vd), _p(o), _p(dd), None, None, Bt2, H2, N, D, 0, BF16, stream)
        assert rc == 7 and "scratch" in ltn.ltn_status_str(rc)  # LTN_ERR_SCRATCH, nothing launched
    finally:
        ltn.ltn_attn_set_debug_plan(0, 0)
