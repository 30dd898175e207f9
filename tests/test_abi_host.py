"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects bad arguments on the
host before anything is launched (no GPU is touched by these calls)."""
import ctypes as C
import os
import re

import pytest

from paper_2511_15927_amd import binding as bd
from paper_2511_15927_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bimamba.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bimamba_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(bd.EXPORTS)
    lib = bd.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert bd.bimamba_version() == 1


def good():
    cfg = synth.mixer_cfg(2, 64, 128, io="bf16")
    desc = bd.make_desc(cfg)
    fake = 0x1000
    p = bd.Params(fake, fake, fake, fake, None)
    t = lambda ch: bd.Tensor(fake, 64 * ch, ch)
    inp = bd.Inputs(t(128), t(128), t(128), t(16), t(16))
    return cfg, desc, p, inp, t(128)


def call_fwd(desc, pf, pb, inp, out, ws=0x1000, ws_bytes=1 << 40):
    return bd.lib().bimamba_fwd(C.byref(desc), C.byref(pf) if pf else None, C.byref(pb) if pb else None,
                                C.byref(inp) if inp else None, None, C.byref(out) if out else None,
                                C.c_void_p(ws), ws_bytes, None)


def test_null_and_shape_errors_are_decided_on_the_host():
    cfg, desc, p, inp, out = good()
    assert call_fwd(desc, None, p, inp, out) == -1
    assert call_fwd(desc, p, p, None, out) == -1
    assert call_fwd(desc, p, p, inp, None) == -1
    assert call_fwd(desc, bd.Params(None, None, 0x1000, 0x1000, None), p, inp, out) == -1
    assert call_fwd(desc, p, p, inp, out, ws=None) == -1
    assert call_fwd(desc, p, p, inp, out, ws_bytes=16) == -5
    assert call_fwd(desc, p, p, inp, out, ws=0x1004) == -4
    bad = bd.Inputs(bd.Tensor(0x1001, 64 * 128, 128), inp.z, inp.dt, inp.B, inp.C)
    assert call_fwd(desc, p, p, bad, out) == -4
    narrow = bd.Inputs(bd.Tensor(0x1000, 64 * 128, 100), inp.z, inp.dt, inp.B, inp.C)
    assert call_fwd(desc, p, p, narrow, out) == -2
    overlap = bd.Inputs(bd.Tensor(0x1000, 128, 128), inp.z, inp.dt, inp.B, inp.C)
    assert call_fwd(desc, p, p, overlap, out) == -2
    wide = bd.Inputs(bd.Tensor(0x1000, 64 * ((1 << 26) + 1), (1 << 26) + 1), inp.z, inp.dt, inp.B, inp.C)
    assert call_fwd(desc, p, p, wide, out) == -3                 # token stride beyond what a tile's 32-bit row offsets reach


def call_bwd(desc, pf, pb, inp, inp_b, dout, gi, gi_b, qf, qb, ws=0x1000, ws_bytes=1 << 40):
    ref = lambda v: C.byref(v) if v is not None else None
    return bd.lib().bimamba_bwd(C.byref(desc), ref(pf), ref(pb), ref(inp), ref(inp_b), ref(dout), ref(gi), ref(gi_b),
                                ref(qf), ref(qb), C.c_void_p(ws), ws_bytes, None)


def test_gradient_call_errors_are_decided_on_the_host():
    cfg, desc, p, inp, dout = good()
    t = lambda ch, at=0x1000: bd.Tensor(at, 64 * ch, ch)
    gi, gi2 = bd.InputGrads(t(128), t(128), t(128), 0x1000, 0x1000), bd.InputGrads(t(128), t(128), t(128), 0x1000, 0x1000)
    qf, qb = bd.ParamGrads(0x1000, None, 0x1000, 0x1000, None), bd.ParamGrads(0x1000, None, 0x1000, 0x1000, None)
    need = bd.bimamba_bwd_workspace_bytes(desc)
    assert need > 0
    assert call_bwd(desc, p, p, inp, None, dout, gi, None, qf, qb, ws_bytes=need - 1) == -5
    assert call_bwd(desc, p, p, inp, None, dout, gi, None, qf, qb, ws=None) == -1
    assert call_bwd(desc, p, p, inp, None, dout, gi, None, qf, qb, ws=0x1008) == -4
    assert call_bwd(desc, None, p, inp, None, dout, gi, None, qf, qb) == -1
    assert call_bwd(desc, p, p, None, None, dout, gi, None, qf, qb) == -1
    assert call_bwd(desc, p, p, inp, None, None, gi, None, qf, qb) == -1
    assert call_bwd(desc, p, p, inp, None, dout, None, None, qf, qb) == -1
    assert call_bwd(desc, p, p, inp, None, dout, gi, None, None, qb) == -1
    assert call_bwd(desc, p, p, inp, None, dout, gi, None, qf, qf) == -8        # the two directions' parameter gradients alias
    # shared activations take one set of input gradients, separate activations need two
    assert call_bwd(desc, p, p, inp, None, dout, gi, gi2, qf, qb) == -1
    other = bd.Inputs(t(128, 0x9000), inp.z, inp.dt, inp.B, inp.C)
    assert call_bwd(desc, p, p, inp, other, dout, gi, None, qf, qb) == -1
    no_db = bd.InputGrads(t(128), t(128), t(128), None, 0x1000)
    assert call_bwd(desc, p, p, inp, None, dout, no_db, None, qf, qb) == -1
    odd = bd.InputGrads(t(128), t(128), t(128), 0x1002, 0x1000)
    assert call_bwd(desc, p, p, inp, None, dout, odd, None, qf, qb) == -4
    narrow = bd.InputGrads(bd.Tensor(0x1000, 64 * 128, 100), t(128), t(128), 0x1000, 0x1000)
    assert call_bwd(desc, p, p, inp, None, dout, narrow, None, qf, qb) == -2
    assert call_bwd(desc, p, p, inp, None, dout, gi, None, bd.ParamGrads(None, None, 0x1000, 0x1000, None), qb) == -1
    # layouts the gradient kernels do not cover are refused, whatever else is passed
    m2 = bd.make_desc(synth.m2_cfg(2, 64, 128, headdim=64, d_state=64))
    assert call_bwd(m2, p, p, inp, None, dout, gi, None, qf, qb) == -3
    assert bd.bimamba_bwd_workspace_bytes(m2) == 0
    n32 = bd.make_desc(synth.mixer_cfg(2, 64, 128, d_state=32))
    assert call_bwd(n32, p, p, inp, None, dout, gi, None, qf, qb) == -3


@pytest.mark.parametrize("field,value,code", [
    ("struct_size", 8, -2), ("batch", -1, -2), ("seqlen", -5, -2), ("d_inner", 0, -2), ("n_heads", 3, -2),
    ("n_groups", 5, -2), ("d_state", 12, -3), ("d_conv", 5, -3), ("d_conv", 0, -2), ("io_dtype", 7, -3),
    ("a_kind", 2, -3), ("d_kind", 9, -3), ("combine", 2, -3), ("dt_softplus", 2, -3), ("conv_bc", -1, -3),
    ("time_chunks", -1, -2), ("state_split", -1, -2), ("state_split", 3, -3), ("state_split", 8, -3),
])
def test_descriptor_validation(field, value, code):
    cfg, desc, p, inp, out = good()
    setattr(desc, field, value)
    assert call_fwd(desc, p, p, inp, out) == code
    assert bd.bimamba_workspace_bytes(desc) == 0
    assert bd.bimamba_time_chunks(desc) == 0


def test_group_tiling_rule():
    cfg = synth.mixer_cfg(1, 8, 96, n_heads=96, n_groups=2)      # 48 channels per group: a wave would straddle groups
    desc = bd.make_desc(cfg)
    assert bd.bimamba_workspace_bytes(desc) == 0


def test_workspace_and_chunk_planning():
    d1 = bd.make_desc(synth.CONFIGS["headline"])
    assert bd.bimamba_time_chunks(d1) == 1                       # chains x 2 lanes per chain already fill the chip
    d2 = bd.make_desc(synth.CONFIGS["cfg2"])
    assert bd.bimamba_time_chunks(d2) == 128                     # batch 1: one lane per chain, 16 waves per SIMD from time segments
    assert bd.bimamba_time_chunks(bd.make_desc(synth.CONFIGS["cfg3_block"])) == 1
    assert bd.bimamba_time_chunks(bd.make_desc(synth.mixer_cfg(1, 100, 64, time_chunks=7))) == 7
    assert bd.bimamba_time_chunks(bd.make_desc(synth.mixer_cfg(1, 5, 64, time_chunks=7))) == 5
    # batch sweep at d_inner 4096 (w = 128 waves per batch element with one lane per chain): whole sequence with two
    # lanes per chain from 1.7 to 5 waves per SIMD (batch 7-20), with one lane per chain above, time segments below
    chunks = {b: bd.bimamba_time_chunks(bd.make_desc(synth.mixer_cfg(b, 8192, 4096))) for b in (1, 4, 6, 7, 8, 12, 16, 20, 21, 24, 64)}
    assert [b for b, n in chunks.items() if n == 1] == [7, 8, 12, 16, 20, 21, 24, 64], chunks
    assert chunks[1] == 32 and chunks[4] == 32 and chunks[6] > 1
    sep = bd.make_desc(synth.mixer_cfg(8, 8192, 4096, combine=1))
    assert bd.bimamba_workspace_bytes(sep) < bd.bimamba_workspace_bytes(d1)     # no partial buffer without ADD
    assert bd.bimamba_workspace_bytes(d1) % 256 == 0


def test_time_parts_of_the_matrix_core_path():
    # 64 heads: batch 1 leaves 3/4 of the CUs empty -> 4 parts; batch 2 -> 2; batch 4 fills the chip -> 1.
    parts = {b: bd.bimamba_time_chunks(bd.make_desc(synth.m2_cfg(b, 8192, 4096))) for b in (1, 2, 3, 4, 8)}
    assert parts == {1: 4, 2: 2, 3: 1, 4: 1, 8: 1}, parts
    # 8 heads: 16 parts at most, and no part shorter than 8 chunks of 64 tokens
    assert bd.bimamba_time_chunks(bd.make_desc(synth.m2_cfg(1, 32768, 512))) == 16
    assert bd.bimamba_time_chunks(bd.make_desc(synth.m2_cfg(1, 2048, 512))) == 4
    assert bd.bimamba_time_chunks(bd.make_desc(synth.m2_cfg(1, 1023, 512))) == 2
    assert bd.bimamba_time_chunks(bd.make_desc(synth.m2_cfg(1, 960, 512))) == 1
    # parts of ceil(chunks / parts) chunks: 17 chunks in 2 parts of 9
    assert bd.bimamba_time_chunks(bd.make_desc(synth.m2_cfg(1, 17 * 64, 512))) == 2
    # the part states live in the workspace
    one = bd.bimamba_workspace_bytes(bd.make_desc(synth.m2_cfg(4, 8192, 4096))) / 4
    assert bd.bimamba_workspace_bytes(bd.make_desc(synth.m2_cfg(1, 8192, 4096))) > one
    # the block variant keeps one part (a block is at most a few chunks)
    assert bd.bimamba_time_chunks(bd.make_desc(synth.m2_cfg(1, 64, 512))) == 1


def test_output_overlapping_an_input_is_rejected_on_the_host():
    """out may not overlap any input view: same buffer in place, a partial overlap, or interleaved columns that collide.
    Column slices of one buffer that stay apart are legal (they are not reached here: a legal call would launch)."""
    cfg, desc, p, inp, out = good()
    Dn, L = 128, 64
    elem = 2
    base = 0x100000
    pitch = 4 * Dn                                                    # one projection buffer, row pitch 512 elements
    col = lambda c, ch: bd.Tensor(base + c * elem, L * pitch, pitch)
    sliced = bd.Inputs(col(0, Dn), col(Dn, Dn), col(2 * Dn, Dn), col(3 * Dn, 16), col(3 * Dn + 16, 16))
    assert call_fwd(desc, p, p, sliced, col(0, Dn)) == -8             # in place over x
    assert call_fwd(desc, p, p, sliced, col(Dn - 1, Dn)) == -8        # columns straddle x and z
    assert call_fwd(desc, p, p, sliced, col(3 * Dn + 8, Dn)) == -8    # wraps over B, C and into the next row's x
    assert call_fwd(desc, p, p, sliced, bd.Tensor(base + (2 * L - 1) * pitch * elem, L * Dn, Dn)) == -8
    # (a column slice of the same buffer that no input uses passes the check: the next error comes from the missing GPU
    # or, on the GPU machine, the call runs; the GPU tests cover that case)
    assert lib_status_alias() == "the output overlaps an input"


def lib_status_alias():
    return bd.lib().bimamba_status_string(-8).decode()


def test_status_strings():
    lib = bd.lib()
    for code in range(0, -9, -1):
        assert lib.bimamba_status_string(code).decode() not in ("", "unknown status")
    assert lib.bimamba_status_string(-99).decode() == "unknown status"
