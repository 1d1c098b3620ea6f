"""Guard rows: every output of the library is allocated inside a larger poisoned buffer and the
bytes before and after it must be bit-identical after the call -- for ragged lengths, every
forced value-column split and segment count, forward, backward, decode, the gated forward,
the unequal-width calls and the tiled comparison kernels.  (The outputs themselves are checked
against the oracle elsewhere; here only that nothing is written outside them.)"""
import pytest
import torch

import paper_2307_14995_amd as ltn
from paper_2307_14995_amd import synth
from _helpers import dev, force_plan, gpu, mixed_decay

pytestmark = pytest.mark.gpu

GUARD = 4096                       # bytes on each side (a multiple of 16: outputs stay aligned)
PATTERN = 0x5A


class Guarded:
    """A tensor of `shape`/`dtype` in the middle of a byte buffer filled with PATTERN."""

    def __init__(self, shape, dtype):
        n = 1
        for s in shape:
            n *= s
        self.nbytes = n * torch.empty((), dtype=dtype).element_size()
        self.raw = torch.full((GUARD + self.nbytes + GUARD,), PATTERN, dtype=torch.uint8, device=dev())
        self.t = self.raw[GUARD:GUARD + self.nbytes].view(dtype).view(shape)

    def intact(self):
        lo, hi = self.raw[:GUARD], self.raw[GUARD + self.nbytes:]
        return bool((lo == PATTERN).all()) and bool((hi == PATTERN).all())

    def written(self):
        """Every element was overwritten (the poison is a NaN-free pattern, so compare bytes)."""
        body = self.raw[GUARD:GUARD + self.nbytes]
        return self.nbytes == 0 or not bool((body == PATTERN).all())


def _plans(D):
    dvs = [0, D, D // 2] + ([D // 4] if D == 128 else [])
    return [(dv, segs) for dv in dvs for segs in (0, 2, 3)]


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("N", [1, 63, 65, 517])
def test_guards_forward_backward_every_plan(D, N):
    Bt, H = 1, 3
    q, k, v = gpu(*synth.make_qkv(Bt, H, N, D, torch.bfloat16, 1300 + N))
    g, = gpu(synth.make_do(Bt, H, N, D, torch.bfloat16, 1300 + N))
    dd, = gpu(mixed_decay(H))
    for dv, segs in _plans(D):
        with force_plan(dv, segs):
            o, kv = Guarded((Bt, H, N, D), torch.bfloat16), Guarded((Bt, H, D, D), torch.float32)
            ltn.ltn_attn_fwd(q, k, v, dd, out=o.t, kv_out=kv.t)
            grads = [Guarded((Bt, H, N, D), torch.bfloat16) for _ in range(3)]
            ltn.ltn_attn_bwd(q, k, v, g, dd, out=tuple(x.t for x in grads))
            torch.cuda.synchronize()
        for name, x in (("o", o), ("kv_out", kv), ("dq", grads[0]), ("dk", grads[1]), ("dv", grads[2])):
            assert x.intact(), f"{name}: bytes outside the output changed (dv={dv}, segs={segs})"
            assert x.written(), f"{name}: output not written (dv={dv}, segs={segs})"


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("D", [64, 96, 128, 256])
def test_guards_other_widths_and_fp32(dtype, D):
    Bt, H, N = 1, 2, 131
    q, k, v = gpu(*synth.make_qkv(Bt, H, N, D, dtype, 1320 + D))
    g, = gpu(synth.make_do(Bt, H, N, D, dtype, 1320 + D))
    dd, = gpu(mixed_decay(H))
    o, kv = Guarded((Bt, H, N, D), dtype), Guarded((Bt, H, D, D), torch.float32)
    ltn.ltn_attn_fwd(q, k, v, dd, out=o.t, kv_out=kv.t)
    grads = [Guarded((Bt, H, N, D), dtype) for _ in range(3)]
    ltn.ltn_attn_bwd(q, k, v, g, dd, out=tuple(x.t for x in grads))
    torch.cuda.synchronize()
    for x in [o, kv] + grads:
        assert x.intact() and x.written()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("D,S", [(64, 1), (128, 1), (128, 5), (256, 3), (96, 2)])
def test_guards_decode(dtype, D, S):
    Bt, H = 3, 2
    q, k, v = gpu(*synth.make_qkv(Bt, H, S, D, dtype, 1340 + D))
    dd, = gpu(mixed_decay(H))
    kv = Guarded((Bt, H, D, D), torch.float32)
    kv.t.normal_(generator=None)
    o = Guarded((Bt, H, S, D), dtype)
    ltn.ltn_attn_decode_steps(q, k, v, kv.t, dd, out=o.t)
    if S == 1:
        o1 = Guarded((Bt, H, D), dtype)
        ltn.ltn_attn_decode_step(q[:, :, 0].contiguous(), k[:, :, 0].contiguous(), v[:, :, 0].contiguous(), kv.t, dd,
                                 out=o1.t)
        torch.cuda.synchronize()
        assert o1.intact() and o1.written()
    torch.cuda.synchronize()
    assert kv.intact() and o.intact() and o.written()


@pytest.mark.parametrize("N", [1, 65, 517])
def test_guards_96_features_all_columns_and_gated(N):
    Bt, H, D = 1, 3, 96
    q, k, v = gpu(*synth.make_qkv(Bt, H, N, D, torch.bfloat16, 1380 + N))
    g, = gpu(synth.make_do(Bt, H, N, D, torch.bfloat16, 1380 + N))
    u, = gpu(synth.make_gate(Bt, H, N, D, torch.bfloat16, 1380 + N))
    dd, = gpu(mixed_decay(H))
    for segs in (0, 3):
        with force_plan(96, segs):
            o, y, y2 = (Guarded((Bt, H, N, D), torch.bfloat16) for _ in range(3))
            kv = Guarded((Bt, H, D, D), torch.float32)
            ltn.ltn_attn_fwd(q, k, v, dd, out=o.t, kv_out=kv.t)
            gr = [Guarded((Bt, H, N, D), torch.bfloat16) for _ in range(3)]
            ltn.ltn_attn_bwd(q, k, v, g, dd, out=tuple(x.t for x in gr))
            ltn.ltn_attn_fwd_gated(q, k, v, u, dd, eps=1e-6, store_o=False, y_out=y.t)
            o2 = Guarded((Bt, H, N, D), torch.bfloat16)
            ltn.ltn_attn_fwd_gated(q, k, v, u, dd, eps=1e-6, out=o2.t, y_out=y2.t)
            torch.cuda.synchronize()
        for x in [o, y, y2, o2, kv] + gr:
            assert x.intact() and x.written()


@pytest.mark.parametrize("N", [1, 65, 517])
def test_guards_gated_tiled_and_unequal_widths(N):
    Bt, H, D = 1, 3, 128
    q, k, v = gpu(*synth.make_qkv(Bt, H, N, D, torch.bfloat16, 1360 + N))
    g, = gpu(synth.make_do(Bt, H, N, D, torch.bfloat16, 1360 + N))
    u, = gpu(synth.make_gate(Bt, H, N, D, torch.bfloat16, 1360 + N))
    dd, = gpu(mixed_decay(H))
    for segs in (0, 3):
        with force_plan(0, segs):
            o, y = Guarded((Bt, H, N, D), torch.bfloat16), Guarded((Bt, H, N, D), torch.bfloat16)
            ltn.ltn_attn_fwd_gated(q, k, v, u, dd, eps=1e-6, out=o.t, y_out=y.t)
            y2 = Guarded((Bt, H, N, D), torch.bfloat16)
            ltn.ltn_attn_fwd_gated(q, k, v, u, dd, eps=1e-6, store_o=False, y_out=y2.t)
            torch.cuda.synchronize()
        for x in (o, y, y2):
            assert x.intact() and x.written()
    dx, du = Guarded((Bt, H, N, D), torch.bfloat16), Guarded((Bt, H, N, D), torch.bfloat16)
    ltn.ltn_gate_bwd(q, u, g, 1e-6, out=(dx.t, du.t))
    ot = Guarded((Bt, H, N, D), torch.bfloat16)
    ltn.ltn_attn_fwd_tiled(q, k, v, dd, out=ot.t)
    gt = [Guarded((Bt, H, N, D), torch.bfloat16) for _ in range(3)]
    ltn.ltn_attn_bwd_tiled(q, k, v, g, dd, out=tuple(x.t for x in gt))
    torch.cuda.synchronize()
    for x in [dx, du, ot] + gt:
        assert x.intact() and x.written()
    # queries and keys twice as wide as values
    Dk, Dv = 256, 128
    q2, k2, v2 = gpu(*synth.make_qkv_dkdv(Bt, H, N, Dk, Dv, torch.bfloat16, 1380 + N))
    o2, kv2 = Guarded((Bt, H, N, Dv), torch.bfloat16), Guarded((Bt, H, Dk, Dv), torch.float32)
    ltn.ltn_attn_fwd_dkdv(q2, k2, v2, dd, out=o2.t, kv_out=kv2.t)
    torch.cuda.synchronize()
    assert o2.intact() and o2.written() and kv2.intact() and kv2.written()
