"""GPU parity of the chunked matrix-core path for the Mamba-2 parameterisation (bf16 I/O, one decay rate per head)
against the fp64 oracle, and against the lane-per-chain kernels it replaces for these shapes."""
import numpy as np
import pytest
import torch

from helpers import assert_close, rel_l2, to_np
from paper_2511_15927_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import gpu_util
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return gpu_util


def case(cfg, seed):
    return synth.make_params(cfg, seed, 0), synth.make_params(cfg, seed, 1), synth.make_inputs(cfg, seed)


@pytest.mark.parametrize("N,P", [(128, 64), (128, 32), (64, 64), (64, 32)])
@pytest.mark.parametrize("L", [1, 40, 64, 65, 200])
def test_ssd_matches_oracle(gpu, oracle, N, P, L):
    cfg = synth.m2_cfg(2, L, 4 * P, headdim=P, d_state=N)
    pf, pb, inp = case(cfg, 1000 + N + P + L)
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp))
    got = gpu.gpu_fwd(cfg, pf, pb, inp)
    assert_close(got, ref, gpu.TOL["bf16"])
    # the lane-per-chain kernels on the same inputs (forced by state_split) agree with the same oracle
    got_valu = gpu.gpu_fwd(cfg, pf, pb, inp, state_split=1)
    assert_close(got_valu, ref, gpu.TOL["bf16"])


@pytest.mark.parametrize("kw", [
    dict(combine=1), dict(conv_bc=0), dict(dt_softplus=0), dict(d_kind=0), dict(d_conv=2), dict(n_groups=2),
    dict(combine=1, conv_bc=0, dt_softplus=0, d_kind=0, d_conv=3),
])
def test_ssd_option_coverage(gpu, oracle, kw):
    cfg = synth.m2_cfg(2, 150, 256, headdim=64, d_state=64, **kw)
    pf, pb, inp = case(cfg, 1100)
    inp_b = synth.make_inputs(cfg, 1101)
    for other in (None, inp_b):
        ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), None if other is None else to_np(other))
        got = gpu.gpu_fwd(cfg, pf, pb, inp, other)
        assert_close(got, ref, gpu.TOL["bf16"], (kw, other is not None))


def test_ssd_long_sequence_state_stays_fp32(gpu, oracle):
    """Many chunks: the state is carried in fp32 accumulators for the whole sequence."""
    cfg = synth.m2_cfg(1, 4096, 256, headdim=64, d_state=128)
    pf, pb, inp = case(cfg, 1200)
    sel = list(range(0, 256, 5))
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), sel=sel)
    got = gpu.gpu_fwd(cfg, pf, pb, inp)[..., sel]
    assert_close(got, ref, gpu.TOL["bf16"])


def test_ssd_block_variant_carries_state_and_tail(gpu, oracle):
    cfg = synth.m2_cfg(2, 96, 128, headdim=32, d_state=64)
    pf, pb, inp = case(cfg, 1300)
    K, Dn, GN = cfg["d_conv"], cfg["d_inner"], cfg["n_groups"] * cfg["d_state"]
    g_full, h_full = oracle.one_direction(cfg, to_np(pf), to_np(inp), +1)
    h, tail = None, None
    h_ref, tail_ref = None, None
    for t0, t1 in ((0, 32), (32, 35), (35, 96)):
        blk = {k: v[:, t0:t1].contiguous() for k, v in inp.items()}
        cb = dict(cfg, seqlen=t1 - t0)
        ref, h_ref, tail_ref = oracle.bimamba_block_fwd(cb, to_np(pf), to_np(pb), to_np(blk), h_in=h_ref, tail_in=tail_ref)
        out, h, tail = gpu.gpu_block_fwd(cb, pf, pb, blk, h_in=h, tail_in=tail)
        assert_close(out, ref, gpu.TOL["bf16"], (t0, t1))
        assert np.array_equal(tail, tail_ref)
        # the chain of GPU states follows the oracle's chain (bf16 operand rounding accumulates only mildly)
        assert rel_l2(h, h_ref) < 1e-2, (t0, t1)
    assert rel_l2(h, h_full) < 1e-2


def test_ssd_benchmark_shapes_sampled(gpu, oracle):
    for name, L in (("cfg1_m2", 2048), ("paper_1p3b", 1024)):
        cfg = dict(synth.CONFIGS[name], batch=2, seqlen=L)
        pf, pb, inp = case(cfg, 1400)
        sel = sorted(np.random.default_rng(3).choice(cfg["d_inner"], size=48, replace=False).tolist())
        ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), sel=sel)
        got = gpu.gpu_fwd(cfg, pf, pb, inp)[..., sel]
        assert_close(got, ref, gpu.TOL["bf16"], name)


@pytest.mark.parametrize("lead", [4, 3])
def test_ssd_strided_views_and_unaligned_fallback(gpu, oracle, lead):
    """Inputs as column slices of one projection buffer.  The chunked kernels read x as channel pairs: with an even
    column offset and even row pitch they run; with an odd offset the call must still succeed (lane-per-chain
    kernels take over inside the same workspace) and give the same answer."""
    from paper_2511_15927_amd import binding as bd
    cfg = synth.m2_cfg(2, 150, 128, headdim=64, d_state=64)
    pf, pb, inp = case(cfg, 1500)
    Bt, L, Dn, H, GN = 2, 150, 128, 2, 64
    widths = dict(z=Dn, x=Dn, B=GN, C=GN, dt=H)
    pitch = lead + sum(widths.values()) + 6
    big = torch.zeros(Bt, L, pitch, dtype=torch.bfloat16, device="cuda")
    views, off = {}, lead
    for k in ("z", "x", "B", "C", "dt"):
        views[k] = big[:, :, off:off + widths[k]]
        views[k].copy_(inp[k].reshape(Bt, L, -1).to(torch.bfloat16))
        off += widths[k]
    assert (views["x"].data_ptr() % 4 == 0) == (lead % 2 == 0)
    desc = bd.make_desc(cfg)
    out_big = torch.zeros(Bt, L, Dn + 8, dtype=torch.bfloat16, device="cuda")
    out = out_big[:, :, 4:4 + Dn]
    dpf, dpb, ws = bd.to_device(pf), bd.to_device(pb), bd.alloc_workspace(desc)
    bd.bimamba_fwd(desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(views), None, bd.make_tensor(out), ws)
    torch.cuda.synchronize()
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp))
    assert_close(out.float().cpu().numpy(), ref, gpu.TOL["bf16"])
    assert torch.all(out_big[:, :, :4] == 0) and torch.all(out_big[:, :, 4 + Dn:] == 0)


@pytest.mark.parametrize("L", [40, 130])
def test_ssd_more_items_than_compute_units(gpu, oracle, L):
    """More (batch, head) pairs than the chip has CUs (several rounds of workgroups), one and three chunks each: the
    full-sequence call, and a block call that loads and commits every pair's state."""
    cfg = synth.m2_cfg(3, L, 32 * 200, headdim=32, d_state=64)       # 600 items, one or three chunks each
    pf, pb, inp = case(cfg, 1600 + L)
    sel = sorted(np.random.default_rng(5).choice(cfg["d_inner"], size=300, replace=False).tolist())
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), sel=sel)
    got = gpu.gpu_fwd(cfg, pf, pb, inp)[..., sel]
    assert_close(got, ref, gpu.TOL["bf16"])
    g = torch.Generator().manual_seed(L)
    h0 = (0.2 * torch.randn(3, cfg["d_inner"], 64, generator=g)).float()
    tail0 = synth.round_io(torch.randn(3, 3, cfg["d_inner"] + 128, generator=g), "bf16")
    ref, h_ref, t_ref = oracle.bimamba_block_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), h_in=h0.numpy(), tail_in=tail0.numpy())
    out, h, tail = gpu.gpu_block_fwd(cfg, pf, pb, inp, h_in=h0, tail_in=tail0)
    assert_close(out, ref, gpu.TOL["bf16"])
    assert rel_l2(h, h_ref) < 1e-2
    assert np.array_equal(tail, t_ref)


def test_ssd_state_not_16_byte_aligned_falls_back(gpu, oracle):
    """The matrix-core kernels move the cached state as 16-byte pieces.  A state buffer that is only 4-byte aligned
    must still work: the call runs on the lane-per-chain kernels inside the same workspace."""
    from paper_2511_15927_amd import binding as bd
    cfg = synth.m2_cfg(2, 70, 128, headdim=64, d_state=64)
    pf, pb, inp = case(cfg, 1700)
    g = torch.Generator().manual_seed(3)
    h0 = (0.2 * torch.randn(2, 128, 64, generator=g)).float()
    ref, h_ref, _ = oracle.bimamba_block_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), h_in=h0.numpy(), want_tail=False)
    n = h0.numel()
    buf_in = torch.zeros(n + 1, dtype=torch.float32, device="cuda")
    buf_out = torch.zeros(n + 1, dtype=torch.float32, device="cuda")
    h_in, h_out = buf_in[1:].view(2, 128, 64), buf_out[1:].view(2, 128, 64)
    h_in.copy_(h0)
    assert h_in.data_ptr() % 16 == 4
    desc = bd.make_desc(cfg)
    dpf, dpb, dinp = bd.to_device(pf), bd.to_device(pb), bd.to_device(inp, cfg)
    out, ws = bd.alloc_out(cfg), bd.alloc_workspace(desc, 1)
    bd.bimamba_block_fwd(desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(dinp), None, h_in, None, h_out,
                         None, bd.make_tensor(out), ws)
    torch.cuda.synchronize()
    assert_close(out.float().cpu().numpy(), ref, gpu.TOL["bf16"])
    assert rel_l2(h_out.cpu().numpy(), h_ref) < 1e-5      # the lane-per-chain kernels keep the state to fp32 accuracy
    assert float(buf_out[0]) == 0.0


@pytest.mark.parametrize("L,batch,N,kw", [(1100, 1, 128, {}), (2117, 2, 64, dict(combine=1)),
                                          (1030, 1, 64, dict(conv_bc=0, dt_softplus=0, d_kind=0))])
def test_ssd_time_parts(gpu, oracle, L, batch, N, kw):
    """Few (batch, head) items and many chunks: each item's chunks are dealt to several workgroups (a state-only pass,
    a carry over the parts, then the output pass).  Ragged last part, both combines, and the block variant: the parts
    start from the cached state and the committed state is the last part's."""
    from paper_2511_15927_amd import binding as bd
    cfg = synth.m2_cfg(batch, L, 256, headdim=64, d_state=N, **kw)
    assert bd.bimamba_time_chunks(bd.make_desc(cfg)) > 1
    pf, pb, inp = case(cfg, 1900 + L)
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp))
    assert_close(gpu.gpu_fwd(cfg, pf, pb, inp), ref, gpu.TOL["bf16"])
    # block variant on top of a prefix
    m = 5
    pre = {k: v[:, :m].contiguous() for k, v in inp.items()}
    blk = {k: v[:, m:].contiguous() for k, v in inp.items()}
    _, h_pre, tail_pre = oracle.bimamba_block_fwd(dict(cfg, seqlen=m), to_np(pf), to_np(pb), to_np(pre))
    cb = dict(cfg, seqlen=L - m)
    assert bd.bimamba_time_chunks(bd.make_desc(cb)) > 1
    ref_b, h_ref, tail_ref = oracle.bimamba_block_fwd(cb, to_np(pf), to_np(pb), to_np(blk), h_in=h_pre.astype(np.float32), tail_in=tail_pre)
    out, h, tail = gpu.gpu_block_fwd(cb, pf, pb, blk, h_in=h_pre.astype(np.float32), tail_in=tail_pre)
    assert_close(out, ref_b, gpu.TOL["bf16"])
    assert rel_l2(h, h_ref) < 1e-2
    assert np.array_equal(tail, tail_ref)


@pytest.mark.parametrize("token_stride", [1 << 24, (1 << 24) + 2])
def test_ssd_time_parts_with_a_wide_x_stride(gpu, oracle, token_stride):
    """x as a view with a token stride of 2^24 elements, the widest for which the state pass of the time parts may
    address a chunk's rows with 32-bit offsets, and just beyond it, where the call runs without parts."""
    from paper_2511_15927_amd import binding as bd
    L = 1030
    cfg = synth.m2_cfg(1, L, 256, headdim=64, d_state=64)
    assert bd.bimamba_time_chunks(bd.make_desc(cfg)) > 1
    pf, pb, inp = case(cfg, 4242)
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp))
    desc = bd.make_desc(cfg)
    dpf, dpb, dinp = bd.to_device(pf), bd.to_device(pb), bd.to_device(inp, cfg)
    big = torch.empty((L - 1) * token_stride + 256, dtype=torch.bfloat16, device="cuda")
    wide = big.as_strided((1, L, 256), (0, token_stride, 1))
    wide.copy_(dinp["x"])
    dinp["x"] = wide
    out, ws = bd.alloc_out(cfg), bd.alloc_workspace(desc)
    bd.bimamba_fwd(desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(dinp), None, bd.make_tensor(out), ws)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    del big, wide, dinp
    torch.cuda.empty_cache()
    assert_close(got, ref, gpu.TOL["bf16"])


@pytest.mark.parametrize("name,batch", [("cfg2_m2", 1), ("headline_m2", 1), ("headline_m2", 2)])
def test_ssd_time_parts_at_benchmark_size_sampled(gpu, oracle, name, batch):
    """The time-part path (state pass over sub-parts, carry, concurrent output pass) at the benchmark's own sizes, in the
    launch configuration the benchmark times; the oracle runs on sampled channels."""
    from paper_2511_15927_amd import binding as bd
    cfg = dict(synth.CONFIGS[name], batch=batch)
    assert bd.bimamba_time_chunks(bd.make_desc(cfg)) > 1
    pf, pb, inp = case(cfg, 1700 + batch)
    sel = sorted(np.random.default_rng(5).choice(cfg["d_inner"], size=24, replace=False).tolist())
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), sel=sel)
    got = gpu.gpu_fwd(cfg, pf, pb, inp)[..., sel]
    assert_close(got, ref, gpu.TOL["bf16"], name)


def test_ssd_block_call_at_benchmark_size_sampled(gpu, oracle):
    """A block-diffusion step at the benchmark's size (batch 16, 32 tokens, 64 heads x 64, N 128) from a cached state and
    conv tail: one scan launch runs both directions of every (batch, head) item; sampled channels against the oracle,
    the committed state of those channels and the whole committed tail."""
    cfg = synth.CONFIGS["cfg3_block_m2"]
    pf, pb, inp = case(cfg, 1800)
    Bt, Dn, N, K = cfg["batch"], cfg["d_inner"], cfg["d_state"], cfg["d_conv"]
    tail_ch = synth.conv_channels(cfg)
    g = torch.Generator().manual_seed(1801)
    h0 = (0.2 * torch.randn(Bt, Dn, N, generator=g)).float()
    tail0 = synth.round_io(torch.randn(Bt, K - 1, tail_ch, generator=g), cfg["io"])
    sel = sorted(np.random.default_rng(6).choice(Dn, size=48, replace=False).tolist())
    ref, h_ref, t_ref = oracle.bimamba_block_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), h_in=h0.numpy(), tail_in=tail0.numpy(), sel=sel)
    out, h, tail = gpu.gpu_block_fwd(cfg, pf, pb, inp, h_in=h0, tail_in=tail0)
    assert_close(out[..., sel], ref, gpu.TOL["bf16"])
    assert rel_l2(h[:, sel, :], h_ref[:, sel, :]) < 1e-2
    assert np.array_equal(tail, t_ref)
