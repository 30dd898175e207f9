"""GPU parity of the sweep in which the lanes of a chain deal the tokens among themselves (two or four lanes per chain,
up to 16 states): forced through state_split so that small shapes reach it, against the fp64 oracle.

What the cases aim at: the hand-over between dealt tiles (8 tokens) and the per-token remainder in both directions and
at the meeting point of the two walks, the conv window across groups, tiles and the cached tail (every conv width), the
per-lane ownership of loads and stores with token strides that differ per tensor, both decay forms, and the committed
state.
"""
import numpy as np
import pytest
import torch

from helpers import assert_close, rel_l2, to_np
from paper_2511_15927_amd import binding as bd
from paper_2511_15927_amd import synth
from test_gpu_block import params, raw_tail

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import gpu_util
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return gpu_util


def forced(cfg, split):
    return dict(cfg, state_split=split, time_chunks=1)


@pytest.mark.parametrize("split", [2, 4])
@pytest.mark.parametrize("L", [8, 15, 16, 17, 31, 32, 33, 47, 64, 203])
def test_lengths_around_whole_tiles(gpu, oracle, split, L):
    """Each direction walks ceil(L/2) or floor(L/2) tokens twice: whole tiles dealt, the rest token by token."""
    for io in ("f32", "bf16"):
        cfg = forced(synth.mixer_cfg(2, L, 72, io=io), split)
        pf, pb = params(cfg, 40 + L, random_a=False)
        inp = synth.make_inputs(cfg, 40 + L)
        got = gpu.gpu_fwd(cfg, pf, pb, inp)
        assert_close(got, oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp)), gpu.TOL[io], cfg)


@pytest.mark.parametrize("split", [2, 4])
@pytest.mark.parametrize("K", [1, 2, 3, 4])
@pytest.mark.parametrize("mode", ["add", "separate", "untied", "softplus", "general_a", "scalar_a"])
def test_modes_and_conv_widths(gpu, oracle, split, K, mode):
    kw = dict(d_conv=K)
    if mode == "separate":
        kw["combine"] = synth.COMBINE_SEPARATE
    if mode == "softplus":
        kw["dt_softplus"] = 1
    if mode == "scalar_a":
        kw.update(n_heads=6, a_kind=synth.A_SCALAR_PER_HEAD, d_kind=synth.D_PER_HEAD)
    cfg = forced(synth.mixer_cfg(2, 77, 96, io="f32", **kw), split)
    pf, pb = params(cfg, 7 * K + split, random_a=mode == "general_a")
    inp = synth.make_inputs(cfg, 5)
    inp_b = synth.make_inputs(cfg, 6) if mode == "untied" else None
    got = gpu.gpu_fwd(cfg, pf, pb, inp, inp_b)
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), None if inp_b is None else to_np(inp_b))
    assert_close(got, ref, gpu.TOL["f32"], cfg)


@pytest.mark.parametrize("split", [2, 4])
def test_progression_decay_bf16(gpu, oracle, split):
    """A = -(1..N): the two-exponential form, whose ratio only the owner of a token evaluates."""
    cfg = forced(synth.mixer_cfg(3, 150, 200, io="bf16"), split)
    pf, pb = params(cfg, 3, random_a=False)
    inp = synth.make_inputs(cfg, 3)
    assert_close(gpu.gpu_fwd(cfg, pf, pb, inp), oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp)), gpu.TOL["bf16"], cfg)


@pytest.mark.parametrize("split", [2, 4])
@pytest.mark.parametrize("K", [2, 4])
def test_block_with_cached_state_and_tail(gpu, oracle, split, K):
    """The forward walk starts from h_in and from a conv window that reaches into tail_in, and commits both."""
    cfg = forced(synth.mixer_cfg(2, 90, 100, io="f32", d_conv=K), split)
    pf, pb = params(cfg, 21)
    inp = synth.make_inputs(cfg, 21)
    m, G = 29, 40
    pre = {k: v[:, :m].contiguous() for k, v in inp.items()}
    blk = {k: v[:, m:m + G].contiguous() for k, v in inp.items()}
    _, h_pre = oracle.one_direction(dict(cfg, seqlen=m), to_np(pf), to_np(pre), +1)
    h_in = h_pre.astype(np.float32)
    tail = raw_tail(cfg, inp, m)
    cb = dict(cfg, seqlen=G)
    ref, h_ref, t_ref = oracle.bimamba_block_fwd(cb, to_np(pf), to_np(pb), to_np(blk), h_in=h_in, tail_in=tail.numpy())
    got, h_got, t_got = gpu.gpu_block_fwd(cb, pf, pb, blk, h_in=h_in, tail_in=tail)
    assert_close(got, ref, gpu.TOL["f32"])
    assert rel_l2(h_got, h_ref) < 1e-5
    assert np.array_equal(t_got, t_ref)


@pytest.mark.parametrize("split", [2, 4])
def test_column_slices_with_their_own_token_strides(gpu, oracle, split):
    """x, z, dt as column slices of one wide buffer, out a slice of another: each tensor has its own row pitch, which is
    what a lane's place inside a tile is computed from."""
    cfg = forced(synth.mixer_cfg(2, 61, 64, io="bf16"), split)
    pf, pb = params(cfg, 9, random_a=False)
    inp = synth.make_inputs(cfg, 9)
    Bt, L, Dn = cfg["batch"], cfg["seqlen"], cfg["d_inner"]
    io = bd.io_dtype(cfg)
    wide = torch.zeros(Bt, L, 3 * Dn + 40, dtype=io, device="cuda")
    wide[..., 8:8 + Dn] = inp["x"].to(io)
    wide[..., 16 + Dn:16 + 2 * Dn] = inp["z"].to(io)
    wide[..., 24 + 2 * Dn:24 + 3 * Dn] = inp["dt"].to(io)
    dev = bd.to_device(inp, cfg)
    views = dict(dev, x=wide[..., 8:8 + Dn], z=wide[..., 16 + Dn:16 + 2 * Dn], dt=wide[..., 24 + 2 * Dn:24 + 3 * Dn])
    out_wide = torch.zeros(Bt, L, Dn + 24, dtype=io, device="cuda")
    out = out_wide[..., 16:16 + Dn]
    desc = bd.make_desc(cfg)
    dpf, dpb = bd.to_device(pf), bd.to_device(pb)
    bd.bimamba_fwd(desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(views), None, bd.make_tensor(out),
                   bd.alloc_workspace(desc))
    torch.cuda.synchronize()
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp))
    assert_close(out.float().cpu().numpy().astype(np.float64), ref, gpu.TOL["bf16"], cfg)
    assert float(out_wide[..., :16].abs().max()) == 0.0 and float(out_wide[..., 16 + Dn:].abs().max()) == 0.0


def test_batch_sixteen_takes_the_dealt_pairs_at_full_length(gpu, oracle):
    """The automatic plan at batch 16, d_inner 4096 (two lanes per chain, two rounds of resident waves), sampled channels."""
    cfg = synth.mixer_cfg(16, 1024, 4096)
    assert bd.bimamba_time_chunks(bd.make_desc(cfg)) == 1
    pf, pb = params(cfg, 77, random_a=False)
    inp = synth.make_inputs(cfg, 77)
    sel = list(range(5, 4096, 409))
    got = gpu.gpu_fwd(cfg, pf, pb, inp)[..., sel]
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), sel=sel)
    assert_close(got, ref, gpu.TOL["bf16"], cfg)
