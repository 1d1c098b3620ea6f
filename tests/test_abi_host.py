"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the public header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2307_14995_amd as ltn
from paper_2307_14995_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ltn_attn.h")

OK, E_NULL, E_SHAPE, E_UNSUP, E_ALIGN, E_DECAY, E_LAUNCH = range(7)
P = 1 << 44  # fake, 16-byte aligned, never dereferenced: validation fails before any launch.
# Fake tensors sit 4 GiB or more apart, so that only the cases that mean to overlap do.


@pytest.fixture(scope="module")
def lib():
    return ltn.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ltn_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    seen = set()
    for code in range(7):
        s = ltn.ltn_status_str(code)
        assert s.startswith("LTN_") and s not in seen
        seen.add(s)
    assert "unknown" in ltn.ltn_status_str(99)


def test_pick_block_and_workspace(lib):
    import torch
    assert ltn.ltn_attn_pick_block(128, torch.bfloat16) == 64
    assert ltn.ltn_attn_pick_block(64, torch.bfloat16) == 64
    assert ltn.ltn_attn_pick_block(64, torch.float32) == 64
    assert ltn.ltn_attn_pick_block(128, torch.float32) == 32
    assert ltn.ltn_attn_pick_block(96, torch.bfloat16) == 64
    assert ltn.ltn_attn_pick_block(96, torch.float32) == 32
    assert ltn.ltn_attn_pick_block(80, torch.bfloat16) == 0
    assert ltn.ltn_attn_pick_block(256, torch.bfloat16) == 64
    assert ltn.ltn_attn_pick_block(256, torch.float32) == 16
    assert ltn.ltn_attn_workspace_bytes(1, 32, 65536, 256, 0, torch.bfloat16, 0) == 0   # 256-wide heads: 4 workgroups per chain already
    assert ltn.ltn_attn_workspace_bytes(1, 8, 65536, 256, 0, torch.bfloat16, 0) == 8 * 8 * 256 * 256 * 4
    assert ltn.ltn_attn_workspace_bytes(1, 8, 65536, 96, 0, torch.bfloat16, 0) == 8 * 10 * 96 * 96 * 4   # three 32-column workgroups per segment
    assert ltn.ltn_attn_workspace_bytes(4, 32, 8192, 128, 0, torch.bfloat16, 1) == 0


def test_check_decay(lib):
    assert ltn.ltn_attn_check_decay([0.0, 0.5, 1.0]) == OK
    assert ltn.ltn_attn_check_decay([0.5, 1.0001]) == E_DECAY
    assert ltn.ltn_attn_check_decay([-1e-9]) == E_DECAY
    assert ltn.ltn_attn_check_decay([float("nan")]) == E_DECAY
    assert lib.ltn_attn_check_decay(None, 3) == E_NULL


def fwd(lib, q=P, k=P + 0x1000000000, v=P + 0x2000000000, o=P + 0x3000000000, decay=P + 0x4000000000, kv_in=None, kv_out=None,
        Bt=1, H=2, N=256, D=64, block=0, dtype=1, ws=None, ws_bytes=0):
    return lib.ltn_attn_fwd(q, k, v, o, decay, kv_in, kv_out, Bt, H, N, D, block, dtype, ws, ws_bytes, None)


def bwd(lib, q=P, k=P + 0x1000000000, v=P + 0x2000000000, g=P + 0x3000000000, dq=P + 0x5000000000, dk=P + 0x6000000000, dv=P + 0x7000000000,
        decay=P + 0x4000000000, Bt=1, H=2, N=256, D=64, block=0, dtype=1):
    return lib.ltn_attn_bwd(q, k, v, g, dq, dk, dv, decay, Bt, H, N, D, block, dtype, None, 0, None)


def test_fwd_argument_errors(lib):
    assert fwd(lib, q=None) == E_NULL
    assert fwd(lib, o=None) == E_NULL
    assert fwd(lib, decay=None) == E_NULL
    assert fwd(lib, N=-1) == E_SHAPE
    assert fwd(lib, Bt=-1) == E_SHAPE
    assert fwd(lib, D=80) == E_UNSUP
    assert fwd(lib, D=96, block=64, dtype=0) == E_UNSUP    # fp32, D = 96 (computed as 128): block <= 32
    assert fwd(lib, D=512) == E_UNSUP
    assert fwd(lib, D=256, block=32, dtype=0) == E_UNSUP   # fp32, D = 256: block 16 only
    assert fwd(lib, D=256, block=32) == E_UNSUP             # bf16: block 64 only
    assert fwd(lib, dtype=7) == E_UNSUP
    assert fwd(lib, block=48) == E_UNSUP
    assert fwd(lib, block=32, dtype=1) == E_UNSUP          # bf16 supports block 64 only
    assert fwd(lib, D=128, block=64, dtype=0) == E_UNSUP   # fp32: D * block <= 4096
    assert fwd(lib, q=P + 8) == E_ALIGN
    assert fwd(lib, kv_out=P + 0x8000000004) == E_ALIGN
    assert fwd(lib, decay=P + 0x4000000002) == E_ALIGN
    assert fwd(lib, o=P) == E_UNSUP                        # output aliases q
    assert fwd(lib, kv_out=P + 0x2000000000) == E_UNSUP          # state aliases v
    # empty problems succeed without touching the GPU
    assert fwd(lib, Bt=0) == OK
    assert fwd(lib, H=0) == OK
    assert fwd(lib, N=0) == OK                             # no state requested -> nothing to do


def test_bwd_argument_errors(lib):
    assert bwd(lib, g=None) == E_NULL
    assert bwd(lib, dv=None) == E_NULL
    assert bwd(lib, N=-5) == E_SHAPE
    assert bwd(lib, D=32) == E_UNSUP
    assert bwd(lib, block=128) == E_UNSUP
    assert bwd(lib, dk=P + 4) == E_ALIGN
    assert bwd(lib, dq=P) == E_UNSUP                       # dq aliases q
    assert bwd(lib, dk=P + 0x5000000000) == E_UNSUP              # dk aliases dq
    assert bwd(lib, Bt=0) == OK
    assert bwd(lib, N=0) == OK


def test_decode_argument_errors(lib):
    f = lib.ltn_attn_decode_step
    args = dict(q=P, k=P + 0x100000000, v=P + 0x200000000, o=P + 0x300000000, kv=P + 0x1000000000, decay=P + 0x4000000000)

    def call(Bt=2, H=2, D=128, dtype=1, **over):
        a = dict(args, **over)
        return f(a["q"], a["k"], a["v"], a["o"], a["kv"], a["decay"], Bt, H, D, dtype, None)

    assert call(kv=None) == E_NULL
    assert call(q=None) == E_NULL
    assert call(Bt=-2) == E_SHAPE
    assert call(D=100) == E_UNSUP
    assert call(dtype=3) == E_UNSUP
    assert call(v=P + 0x200000002) == E_ALIGN
    assert call(o=P + 0x100000000) == E_UNSUP
    assert call(Bt=0) == OK


def test_decode_steps_argument_errors(lib):
    f = lib.ltn_attn_decode_steps

    def call(q=P, k=P + 0x1000000000, v=P + 0x2000000000, o=P + 0x3000000000, kv=P + 0x10000000000, decay=P + 0x4000000000,
             Bt=2, H=2, S=4, D=128, dtype=1):
        return f(q, k, v, o, kv, decay, Bt, H, S, D, dtype, None)

    assert call(kv=None) == E_NULL
    assert call(S=-1) == E_SHAPE
    assert call(D=80) == E_UNSUP
    assert call(q=P + 2) == E_ALIGN
    assert call(o=P + 0x2000000000) == E_UNSUP                   # o aliases v
    assert call(S=0) == OK
    assert call(S=0, q=None, k=None, v=None, o=None) == OK # nothing to read: pointers may be NULL


def test_public_header_is_plain_c_and_cxx(tmp_path):
    """The boundary is a C ABI: the header must compile on its own as C99 and as C++ (no torch or
    HIP types in the signatures)."""
    import os
    import shutil
    import subprocess
    hdr = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "ltn_attn.h")
    for cc, args in (("gcc", ["-xc", "-std=c99"]), ("g++", ["-xc++", "-std=c++17"])):
        if shutil.which(cc) is None:
            pytest.skip(cc + " not available")
        r = subprocess.run([cc] + args + ["-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", hdr],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_fwd_gated_argument_errors(lib):
    f = lib.ltn_attn_fwd_gated
    cf = ctypes.c_float

    def call(q=P, k=P + 0x1000000000, v=P + 0x2000000000, u=P + 0x3000000000, o=P + 0x5000000000, y=P + 0x6000000000, decay=P + 0x4000000000,
             kv_in=None, kv_out=None, eps=1e-6, Bt=1, H=2, N=256, D=64, block=0, dtype=1):
        return f(q, k, v, u, o, y, decay, kv_in, kv_out, cf(eps), Bt, H, N, D, block, dtype, None, 0, None)

    assert call(u=None) == E_NULL
    assert call(y=None) == E_NULL
    assert call(eps=-1.0) == E_SHAPE
    assert call(eps=float("nan")) == E_SHAPE
    assert call(D=96, o=None, dtype=0) == E_UNSUP          # 96 features in fp32, 256 features: only with the attention
    assert call(D=256, o=None) == E_UNSUP                  # output stored (no kernel holds a complete row there)
    assert call(D=80) == E_UNSUP
    assert call(y=P + 0x3000000000) == E_UNSUP                   # y aliases the gate
    assert call(y=P + 0x5000000000) == E_UNSUP                   # y aliases o
    assert call(u=P + 0x3000000008) == E_ALIGN
    assert call(N=0) == OK
    assert call(Bt=0, q=None, k=None, v=None, u=None, o=None, y=None) == OK


def test_fwd_tiled_argument_errors(lib):
    f = lib.ltn_attn_fwd_tiled

    def call(q=P, k=P + 0x1000000000, v=P + 0x2000000000, o=P + 0x3000000000, decay=P + 0x4000000000, Bt=1, H=2, N=256, D=128, dtype=1):
        return f(q, k, v, o, decay, Bt, H, N, D, dtype, None)

    assert call(o=None) == E_NULL
    assert call(N=-1) == E_SHAPE
    assert call(dtype=0) == E_UNSUP                        # bf16 only
    assert call(D=96) == E_UNSUP
    assert call(k=P + 0x1000000002) == E_ALIGN
    assert call(o=P + 0x1000000000) == E_UNSUP                   # o aliases k
    assert call(N=0) == OK


def test_bwd_tiled_argument_errors(lib):
    f = lib.ltn_attn_bwd_tiled

    def call(q=P, k=P + (1 << 36), v=P + (2 << 36), g=P + (3 << 36), dq=P + (5 << 36), dk=P + (6 << 36),
             dv=P + (7 << 36), decay=P + (4 << 36), Bt=1, H=2, N=256, D=128, dtype=1):
        return f(q, k, v, g, dq, dk, dv, decay, Bt, H, N, D, dtype, None)

    assert call(g=None) == E_NULL and call(dq=None) == E_NULL and call(decay=None) == E_NULL
    assert call(N=-1) == E_SHAPE
    assert call(dtype=0) == E_UNSUP                        # bf16 only
    assert call(D=96) == E_UNSUP
    assert call(dk=P + (6 << 36) + 2) == E_ALIGN
    assert call(dv=P + (2 << 36) + 64) == E_UNSUP          # dv starts inside v
    assert call(N=0) == OK and call(Bt=0) == OK


def test_gate_argument_errors(lib):
    cf = ctypes.c_float
    fw, bw = lib.ltn_gate_fwd, lib.ltn_gate_bwd
    assert fw(None, P + 0x1000000000, P + 0x2000000000, cf(0.0), 16, 128, 1, None) == E_NULL
    assert fw(P, P + 0x1000000000, P + 0x2000000000, cf(0.0), -1, 128, 1, None) == E_SHAPE
    assert fw(P, P + 0x1000000000, P + 0x2000000000, cf(-0.5), 16, 128, 1, None) == E_SHAPE
    assert fw(P, P + 0x1000000000, P + 0x2000000000, cf(0.0), 16, 80, 1, None) == E_UNSUP
    assert fw(P, P + 0x1000000000, P + 0x2000000000, cf(0.0), 16, 128, 5, None) == E_UNSUP
    assert fw(P, P + 0x1000000000, P, cf(0.0), 16, 128, 1, None) == E_UNSUP              # y aliases x
    assert fw(P, P + 0x1000000004, P + 0x2000000000, cf(0.0), 16, 128, 1, None) == E_ALIGN
    assert fw(None, None, None, cf(0.0), 0, 128, 1, None) == OK                     # no rows
    assert bw(P, P + 0x1000000000, None, P + 0x3000000000, P + 0x4000000000, cf(0.0), 16, 128, 1, None) == E_NULL
    assert bw(P, P + 0x1000000000, P + 0x2000000000, P + 0x3000000000, P + 0x3000000000, cf(0.0), 16, 128, 1, None) == E_UNSUP  # d_x aliases d_u
    assert bw(P, P + 0x1000000000, P + 0x2000000000, P + 0x3000000000, P + 0x4000000000, cf(0.0), 16, 64, 7, None) == E_UNSUP


def test_dkdv_argument_errors(lib):
    def f(q=P, k=P + 0x1000000000, v=P + 0x2000000000, o=P + 0x3000000000, decay=P + 0x4000000000, kv_in=None, kv_out=None,
          Bt=1, H=2, N=256, Dk=256, Dv=128, block=0, dtype=1):
        return lib.ltn_attn_fwd_dkdv(q, k, v, o, decay, kv_in, kv_out, Bt, H, N, Dk, Dv, block, dtype, None, 0, None)
    assert f(q=None) == E_NULL and f(o=None) == E_NULL and f(decay=None) == E_NULL
    assert f(N=-1) == E_SHAPE and f(Dk=0) == E_SHAPE
    assert f(Dk=128, Dv=128) == E_UNSUP            # equal widths: the plain entry points
    assert f(Dk=256, Dv=64) == E_UNSUP and f(Dk=64, Dv=128) == E_UNSUP
    assert f(dtype=7) == E_UNSUP
    assert f(block=32) == E_UNSUP                  # bf16: 64 only
    assert f(dtype=0, block=32) == E_UNSUP         # fp32 with 256-wide keys: 16 only
    assert f(dtype=0, Dk=128, Dv=64, block=64) == E_UNSUP
    assert f(q=P + 8) == E_ALIGN and f(kv_in=P + 4) == E_ALIGN
    assert f(o=P) == E_UNSUP                       # output aliases q
    assert f(q=None, k=None, v=None, o=None, N=0) == OK
    assert f(Bt=0) == OK

    def b(q=P, k=P + 0x1000000000, v=P + 0x2000000000, g=P + 0x3000000000, dq=P + 0x5000000000, dk=P + 0x6000000000, dv=P + 0x7000000000,
          decay=P + 0x4000000000, Bt=1, H=2, N=256, Dk=256, Dv=128, block=0, dtype=1):
        return lib.ltn_attn_bwd_dkdv(q, k, v, g, dq, dk, dv, decay, Bt, H, N, Dk, Dv, block, dtype, None, 0, None)
    assert b(g=None) == E_NULL and b(dk=None) == E_NULL
    assert b(Dk=128, Dv=128) == E_UNSUP and b(N=-2) == E_SHAPE
    assert b(dq=P) == E_UNSUP and b(dk=P + 0x7000000000) == E_UNSUP
    assert b(dv=P + 0x7000000008) == E_ALIGN
    assert b(N=0) == OK

    # few long chains: the unequal-width calls are cut into segments too and then need their workspace
    import torch
    assert ltn.ltn_attn_workspace_bytes_dkdv(4, 32, 8192, 256, 128, torch.bfloat16, 0) == 0
    need = ltn.ltn_attn_workspace_bytes_dkdv(1, 8, 16384, 256, 128, torch.bfloat16, 0)
    assert need == 8 * 16 * 256 * 128 * 4                  # 16 segments of 1024 tokens, two 64-column workgroups each
    assert ltn.ltn_attn_workspace_bytes_dkdv(1, 8, 16384, 256, 128, torch.float32, 0) == 0
    assert ltn.ltn_attn_workspace_bytes_dkdv(1, 8, 16384, 256, 128, torch.bfloat16, 1) >= need
    assert ltn.ltn_attn_workspace_bytes_dkdv(1, 8, 16384, 128, 128, torch.bfloat16, 0) == 0   # no such shape
    assert f(H=8, N=16384) == E_SHAPE                      # workspace too small
    assert lib.ltn_attn_fwd_dkdv(P, P + (1 << 36), P + (2 << 36), P + (3 << 36), P + (4 << 36), None, None,
                                 1, 8, 16384, 256, 128, 0, 1, None, need, None) == E_NULL

    def d(q=P, k=P + 0x1000000000, v=P + 0x2000000000, o=P + 0x3000000000, kv=P + 0x8000000000, decay=P + 0x4000000000,
          Bt=1, H=2, S=3, Dk=256, Dv=128, dtype=1):
        return lib.ltn_attn_decode_steps_dkdv(q, k, v, o, kv, decay, Bt, H, S, Dk, Dv, dtype, None)
    assert d(kv=None) == E_NULL and d(S=-1) == E_SHAPE and d(Dk=128, Dv=128) == E_UNSUP
    assert d(kv=P + 0x3000000000) == E_UNSUP and d(o=P + 2) == E_ALIGN
    assert d(S=0, q=None, k=None, v=None, o=None, kv=None) == OK


def test_prologue_argument_errors(lib):
    def f(x=P, theta=P + 0x4000000000, y=P + 0x1000000000, act=1, Bt=1, H=2, N=100, D=128, pos0=0, dtype=1):
        return lib.ltn_prologue_fwd(x, theta, y, act, Bt, H, N, D, pos0, dtype, None)
    assert f(x=None) == E_NULL and f(y=None) == E_NULL
    assert f(N=-1) == E_SHAPE and f(pos0=-1) == E_SHAPE and f(pos0=1 << 41) == E_SHAPE
    assert f(D=96) == E_UNSUP and f(dtype=3) == E_UNSUP
    assert f(x=P + 2) == E_ALIGN and f(theta=P + 0x4000000002) == E_ALIGN
    assert f(y=P) == E_UNSUP                       # output aliases the input
    assert f(N=0, x=None, y=None) == OK

    def b(x=P, theta=P + 0x4000000000, dy=P + 0x1000000000, dx=P + 0x2000000000, dth=P + 0x5000000000, act=1, Bt=1, H=2, N=100, D=128,
          pos0=0, dtype=1, ws=P + 0x9000000000, ws_bytes=1 << 20):
        return lib.ltn_prologue_bwd(x, theta, dy, dx, dth, act, Bt, H, N, D, pos0, dtype, ws, ws_bytes, None)
    assert b(dy=None) == E_NULL and b(dx=None) == E_NULL
    assert b(theta=None) == E_NULL                 # an angle gradient without angles
    assert b(ws=None) == E_NULL and b(ws_bytes=16) == E_SHAPE
    assert b(dx=P) == E_UNSUP and b(dth=P + 0x1000000000) == E_UNSUP
    assert b(dth=P + 0x5000000002) == E_ALIGN
    need = lib.ltn_prologue_workspace_bytes(1, 2, 100, 128)
    assert need == 2 * 2 * 128 * 8                 # two 64-token chunks x H x D doubles
    assert b(ws_bytes=need - 1) == E_SHAPE
    assert lib.ltn_prologue_workspace_bytes(1, 2, 0, 128) == 0


def test_partial_overlap_is_refused(lib):
    """Aliasing is judged on byte ranges, not base pointers: an output that starts inside an
    input (or inside another output, or the workspace inside a tensor) is refused."""
    tb = 1 * 2 * 256 * 64 * 2                      # bytes of one [1,2,256,64] bf16 tensor
    assert fwd(lib, o=P + 128) == E_UNSUP          # o starts inside q
    assert fwd(lib, o=P + tb - 16) == E_UNSUP      # o's first row is q's last
    assert fwd(lib, o=P + tb) == OK or fwd(lib, o=P + tb) == E_LAUNCH   # adjacent is fine (fake pointers: no GPU here)
    assert bwd(lib, dk=P + 0x50_0000_0000 + 64) == E_UNSUP   # dk inside dq
    assert bwd(lib, dv=P + 0x20_0000_0000 - 16) == E_UNSUP   # dv's tail reaches into v
    f = lib.ltn_attn_decode_steps
    assert f(P, P + (1 << 32), P + (2 << 32), P + (3 << 32), P + (3 << 32) + 256, P + (9 << 32), 2, 2, 4, 128, 1, None) == E_UNSUP
    # kv_out == kv_in is the one allowed alias; a shifted overlap of the two is not
    assert fwd(lib, kv_in=P + (7 << 32), kv_out=P + (7 << 32) + 4096) == E_UNSUP


def test_debug_plan_and_plan_query(lib):
    import torch
    assert lib.ltn_attn_set_debug_plan(48, 0) == E_SHAPE
    assert lib.ltn_attn_set_debug_plan(0, -1) == E_SHAPE
    assert lib.ltn_attn_set_debug_plan(0, 5000) == E_SHAPE
    assert ltn.ltn_attn_query_plan(4, 32, 8192, 128, torch.bfloat16, 0) == (64, 1)    # headline forward: two slices
    assert ltn.ltn_attn_query_plan(4, 32, 8192, 128, torch.bfloat16, 1) == (128, 1)   # headline backward: full width
    assert ltn.ltn_attn_query_plan(1, 2, 8192, 128, torch.bfloat16, 0) == (32, 16)      # 32 chain segments of 512 tokens, four slices each
    # backward of 4 chains: 21 ways would fill the chip, 20 keeps chains x segments a multiple of 8
    assert ltn.ltn_attn_query_plan(1, 4, 32768, 128, torch.bfloat16, 1) == (128, 20)
    assert ltn.ltn_attn_query_plan(1, 12, 16384, 128, torch.bfloat16, 1) == (128, 6)
    assert ltn.ltn_attn_query_plan(1, 4, 32768, 128, torch.bfloat16, 0) == (128, 64)
    # heads of 96 features: three-slice segments stay within an XCD's 32 units (80 chain segments,
    # not 84); from 12 chain passes on the cut is made for one 96-column workgroup per segment
    assert ltn.ltn_attn_query_plan(1, 4, 32768, 96, torch.bfloat16, 0) == (32, 20)
    assert ltn.ltn_attn_query_plan(1, 32, 8192, 96, torch.bfloat16, 0) == (96, 8)
    assert ltn.ltn_attn_query_plan(1, 32, 2048, 96, torch.bfloat16, 0) == (32, 1)
    assert ltn.ltn_attn_query_plan(1, 16, 8192, 96, torch.bfloat16, 1) == (96, 5)
    assert ltn.ltn_attn_query_plan(1, 16, 4096, 96, torch.bfloat16, 1) == (32, 1)
    # slices of a chain share an XCD's L2 only when an XCD's share of workgroups fits its 32 units:
    # 20 chains backward, 3 passes x 4 slices x 3 chains per XCD = 36 -> two slices per pass instead
    assert ltn.ltn_attn_query_plan(1, 20, 4096, 128, torch.bfloat16, 1) == (64, 1)
    assert ltn.ltn_attn_query_plan(1, 16, 4096, 128, torch.bfloat16, 1) == (32, 1)
    assert ltn.ltn_attn_query_plan(1, 42, 4096, 128, torch.bfloat16, 1) == (128, 1)
    assert ltn.ltn_attn_query_plan(1, 80, 4096, 96, torch.bfloat16, 0) == (32, 1)     # 10 chains x 3 slices per XCD
    assert ltn.ltn_attn_query_plan(1, 82, 4096, 96, torch.bfloat16, 0) == (96, 1)     # 11 would not fit its 32 units
    try:
        ltn.ltn_attn_set_debug_plan(32, 3)
        assert ltn.ltn_attn_query_plan(4, 32, 8192, 128, torch.bfloat16, 0) == (32, 3)
        assert ltn.ltn_attn_workspace_bytes(4, 32, 8192, 128, 0, torch.bfloat16, 0) == 128 * 3 * 128 * 128 * 4
    finally:
        ltn.ltn_attn_set_debug_plan(0, 0)
    assert ltn.ltn_attn_workspace_bytes(4, 32, 8192, 128, 0, torch.bfloat16, 0) == 0
    dv, segs = ctypes.c_int(), ctypes.c_int()
    assert lib.ltn_attn_query_plan(1, 1, 64, 128, 1, 0, None, ctypes.byref(segs)) == E_NULL
    assert lib.ltn_attn_query_plan(1, 1, 64, 80, 1, 0, ctypes.byref(dv), ctypes.byref(segs)) == E_UNSUP
    assert lib.ltn_attn_query_plan(1, 1, 64, 128, 1, 7, ctypes.byref(dv), ctypes.byref(segs)) == E_SHAPE


def test_environment_does_not_change_the_plan(lib, monkeypatch):
    import torch
    monkeypatch.setenv("LTN_ATTN_DV", "32")
    monkeypatch.setenv("LTN_ATTN_SEGS", "5")
    assert ltn.ltn_attn_query_plan(4, 32, 8192, 128, torch.bfloat16, 0) == (64, 1)
    assert ltn.ltn_attn_workspace_bytes(4, 32, 8192, 128, 0, torch.bfloat16, 0) == 0


def test_probe_argument_errors(lib):
    f = lib.ltn_probe_stream_read
    big = 256 * (16 << 20)
    assert f(None, big, 65536, 4, 1, 0, P + 64, None) == E_NULL
    assert f(P, big, 65536, 4, 1, 0, None, None) == E_NULL
    assert f(P, big, 1000, 4, 1, 0, P + (1 << 36), None) == E_SHAPE           # not a multiple of 64 KB
    assert f(P, 65536 * 4 - 1, 65536, 4, 1, 0, P + (1 << 36), None) == E_SHAPE  # regions would leave the buffer
    assert f(P, big, 65536, 0, 1, 0, P + (1 << 36), None) == E_SHAPE
    assert f(P + 4, big, 65536, 4, 1, 0, P + (1 << 36), None) == E_ALIGN


def test_workspace_query(lib):
    import torch
    D = 128
    # few long chains: one fp32 state per (pass, chain, segment); 16 segments of 512 tokens here
    assert ltn.ltn_attn_workspace_bytes(1, 2, 8192, D, 0, torch.bfloat16, 0) == 1 * 2 * 16 * D * D * 4
    assert ltn.ltn_attn_workspace_bytes(1, 2, 8192, D, 0, torch.bfloat16, 1) == 3 * 2 * 16 * D * D * 4
    assert ltn.ltn_attn_workspace_bytes(1, 2, 8192, D, 0, torch.float32, 0) == 0     # bf16 kernels only
    assert ltn.ltn_attn_workspace_bytes(1, 32, 4096, D, 0, torch.bfloat16, 0) == 32 * 8 * D * D * 4   # 8 segments of 512 tokens
    assert ltn.ltn_attn_workspace_bytes(1, 32, 2048, D, 0, torch.bfloat16, 0) == 0   # segments would be too short
    assert ltn.ltn_attn_workspace_bytes(1, 64, 16384, D, 0, torch.bfloat16, 0) == 0  # 4 segments at most: not worth it
    # 5 .. 7 segments only when they are long: the backward of 16 chains (48 passes)
    assert ltn.ltn_attn_workspace_bytes(1, 16, 16384, D, 0, torch.bfloat16, 1) == 3 * 16 * 5 * D * D * 4
    assert ltn.ltn_attn_workspace_bytes(1, 16, 8192, D, 0, torch.bfloat16, 1) == 3 * 16 * 5 * D * D * 4   # 1638 tokens each
    assert ltn.ltn_attn_workspace_bytes(1, 16, 4096, D, 0, torch.bfloat16, 1) == 0     # 819 tokens each: too short
    assert ltn.ltn_attn_query_plan(1, 40, 8192, D, torch.bfloat16, 0) == (128, 6)      # forward of 40 chains: 6 ways
    assert ltn.ltn_attn_query_plan(1, 40, 4096, D, torch.bfloat16, 0) == (32, 1)
    # 4 ways: the backward alone, chains x 4 a multiple of 8, segments of at least 2048 tokens
    assert ltn.ltn_attn_query_plan(1, 20, 8192, D, torch.bfloat16, 1) == (128, 4)
    assert ltn.ltn_attn_query_plan(1, 21, 8192, D, torch.bfloat16, 1) == (64, 1)
    assert ltn.ltn_attn_query_plan(1, 20, 4096, D, torch.bfloat16, 1) == (64, 1)
    assert ltn.ltn_attn_query_plan(1, 60, 8192, D, torch.bfloat16, 0) == (32, 1)
    assert ltn.ltn_attn_workspace_bytes(0, 2, 8192, D, 0, torch.bfloat16, 0) == 0
    # the gated forward keeps full-width slices, so it cuts chains sooner (from 4 segments on, or 2 long ones)
    # (8 segments of 512 tokens, as its other form, plain forward + gate kernel, takes: room for either)
    assert ltn.ltn_attn_query_plan(1, 32, 4096, D, torch.bfloat16, 2) == (128, 8)
    assert ltn.ltn_attn_workspace_bytes(1, 32, 4096, D, 0, torch.bfloat16, 2) == 32 * 8 * D * D * 4
    for (Bt, H, N) in [(1, 2, 2048), (1, 4, 4096), (1, 8, 8192), (2, 8, 16384), (1, 32, 65536), (1, 48, 16384), (4, 32, 8192)]:
        for d in (64, 96, 128, 256):
            assert ltn.ltn_attn_workspace_bytes(Bt, H, N, d, 0, torch.bfloat16, 2) >= \
                ltn.ltn_attn_workspace_bytes(Bt, H, N, d, 0, torch.bfloat16, 0)
    assert ltn.ltn_attn_workspace_bytes(4, 32, 8192, D, 0, torch.bfloat16, 2) == 0
    assert ltn.ltn_attn_workspace_bytes(1, 2, 8192, D, 0, torch.bfloat16, 3) == 0     # no such call


def test_binding_rejects_cpu_tensors():
    import torch
    x = torch.zeros(1, 1, 4, 64)
    with pytest.raises(ValueError):
        ltn.ltn_attn_fwd(x, x, x, torch.ones(1))


def test_product_path_does_not_import_the_oracle():
    """The library's Python side must never reach into oracle/ (and vice versa)."""
    pkg_dir = os.path.join(ROOT, "paper_2307_14995_amd")
    for dirpath, _, files in os.walk(pkg_dir):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("the cpu oracle's tests", ""), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2307_14995_amd" not in text and "libltn_attn" not in text, f


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU measurement: any other --gpus value exits with a message, before
    anything touches a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
