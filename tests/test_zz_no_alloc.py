"""bimamba_block_fwd_static (the block step on the library's own fixed scratch buffer, for callers that cannot
allocate) against bimamba_block_fwd on a caller-provided workspace: same kernels, so outputs, committed state and
committed conv tail must be bit-identical.  Two calls in a row share the buffer, the second with a smaller input."""
import pytest
import torch

from paper_2511_15927_amd import synth

pytestmark = pytest.mark.gpu


def both_ways(bd, cfg, seed):
    """One committing block call from a cached state and conv tail, through both entry points."""
    N, K, Bt, Dn = cfg["d_state"], cfg["d_conv"], cfg["batch"], cfg["d_inner"]
    tail_ch = synth.conv_channels(cfg)
    pf, pb = synth.make_params(cfg, seed, 0), synth.make_params(cfg, seed, 1)
    dpf, dpb = bd.to_device(pf), bd.to_device(pb)
    cpf, cpb = bd.make_params(dpf), bd.make_params(dpb)
    dinp = bd.to_device(synth.make_inputs(cfg, seed), cfg)
    cin = bd.make_inputs(dinp)
    g = torch.Generator().manual_seed(seed)
    h_in = (0.2 * torch.randn(Bt, Dn, N, generator=g)).float().cuda()
    tail_in = torch.randn(Bt, K - 1, tail_ch, generator=g).to(bd.io_dtype(cfg)).cuda()
    desc = bd.make_desc(cfg)
    res = []
    for static in (False, True):
        out = torch.full((Bt, cfg["seqlen"], Dn), float("nan"), dtype=bd.io_dtype(cfg), device="cuda")
        h_out = torch.full_like(h_in, float("nan"))
        tail_out = torch.full_like(tail_in, float("nan"))
        if static:
            bd.bimamba_block_fwd_static(desc, cpf, cpb, cin, None, h_in, tail_in, h_out, tail_out, bd.make_tensor(out))
        else:
            ws = bd.alloc_workspace(desc, 1)
            bd.bimamba_block_fwd(desc, cpf, cpb, cin, None, h_in, tail_in, h_out, tail_out, bd.make_tensor(out), ws)
        torch.cuda.synchronize()
        res.append((out, h_out, tail_out))
    (o0, h0, t0), (o1, h1, t1) = res
    assert not torch.isnan(o0.float()).any() and not torch.isnan(h0).any()
    assert torch.equal(o0, o1) and torch.equal(h0, h1) and torch.equal(t0, t1), cfg


@pytest.mark.parametrize("layout", ["selective", "mamba2"])
def test_static_scratch_block_step_equals_workspace_call(layout):
    from paper_2511_15927_amd import binding as bd
    assert torch.cuda.is_available(), "these tests need the MI355X"
    if layout == "selective":
        first, second = synth.mixer_cfg(4, 96, 1024), synth.mixer_cfg(2, 32, 320)     # 96 tokens: prepared B|C rows + partial
    else:
        first, second = synth.m2_cfg(4, 130, 512, headdim=64, d_state=128), synth.m2_cfg(3, 32, 256, headdim=32, d_state=64)
    assert 0 < bd.bimamba_workspace_bytes(bd.make_desc(second), 1) < bd.bimamba_workspace_bytes(bd.make_desc(first), 1)
    both_ways(bd, first, 71)
    both_ways(bd, second, 72)        # a smaller call over the contents the first one left in the buffer
    both_ways(bd, first, 73)


def test_static_scratch_rejects_calls_beyond_its_size():
    from paper_2511_15927_amd import binding as bd
    assert torch.cuda.is_available(), "these tests need the MI355X"
    cfg = synth.mixer_cfg(16, 512, 4096)        # the fp32 partial alone is 128 MiB
    desc = bd.make_desc(cfg)
    assert bd.bimamba_workspace_bytes(desc, 1) > bd.STATIC_SCRATCH_BYTES
    pf = synth.make_params(cfg, 1, 0)
    dpf = bd.to_device(pf)
    cp = bd.make_params(dpf)
    t = torch.zeros(1, 1, 1, dtype=torch.bfloat16, device="cuda")
    fake = bd.Tensor(t.data_ptr(), 512 * 4096, 4096)
    ins = bd.Inputs(fake, fake, fake, bd.Tensor(t.data_ptr(), 512 * 16, 16), bd.Tensor(t.data_ptr(), 512 * 16, 16))
    rc = bd.bimamba_block_fwd_static(desc, cp, cp, ins, None, None, None, None, None, fake, check=False)
    assert rc == -7 and "scratch" in bd.lib().bimamba_status_string(rc).decode()
