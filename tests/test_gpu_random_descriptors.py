"""GPU parity over seeded random descriptors: shapes, layouts, modes and launch overrides drawn at random (fixed seeds)
from the supported space, every draw checked element by element against the fp64 oracle, full-sequence and block
entry points alike.  Complements the hand-picked cases of the other GPU test files."""
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


def draw(rng):
    """One supported descriptor plus call options."""
    layout = rng.choice(["selective", "heads", "mamba2_valu", "mamba2_mfma"])
    io = "bf16" if layout == "mamba2_mfma" else rng.choice(["f32", "bf16"])
    K = int(rng.integers(1, 5))
    L = int(rng.choice([1, 2, 5, 31, 64, 65, 97, 130, 257]))
    Bt = int(rng.integers(1, 4))
    kw = dict(d_conv=K, io=io, combine=int(rng.integers(0, 2)))
    if layout == "selective":
        N = int(rng.choice([4, 8, 16, 32]))
        Dn = int(rng.choice([1, 7, 64, 100, 192]))
        cfg = synth.mixer_cfg(Bt, L, Dn, d_state=N, dt_softplus=int(rng.integers(0, 2)), **kw)
    elif layout == "heads":
        N = int(rng.choice([16, 32, 64]))
        P = int(rng.choice([8, 64]))
        G = int(rng.choice([1, 2]))
        H = 2 * G * int(rng.integers(1, 3))
        if G > 1:
            P = 64
        cfg = synth.mixer_cfg(Bt, L, H * P, d_state=N, n_heads=H, n_groups=G, a_kind=int(rng.integers(0, 2)),
                              d_kind=int(rng.integers(0, 2)), dt_softplus=int(rng.integers(0, 2)),
                              conv_bc=int(rng.integers(0, 2)), **kw)
    else:
        N = int(rng.choice([64, 128]))
        P = int(rng.choice([32, 64]))
        H = int(rng.integers(1, 4))
        cfg = synth.m2_cfg(Bt, L, H * P, headdim=P, d_state=N, **kw)
        if layout == "mamba2_valu":
            cfg["state_split"] = int(rng.choice([1, 4]))
    if layout != "mamba2_mfma" and L >= 31 and rng.integers(0, 2):
        cfg["time_chunks"] = int(rng.integers(2, 5))
    untied = bool(rng.integers(0, 2))
    random_a = bool(rng.integers(0, 2))
    if layout == "mamba2_mfma" and rng.integers(0, 3) == 0:
        # long enough for the chunked kernels to deal a head's chunks to several workgroups (time parts)
        cfg["seqlen"] = int(rng.choice([1030, 1280, 2117]))
    return layout, cfg, untied, random_a


@pytest.mark.parametrize("seed", range(96))
def test_random_descriptor(gpu, oracle, seed):
    rng = np.random.default_rng(9000 + seed)
    layout, cfg, untied, random_a = draw(rng)
    pf, pb = synth.make_params(cfg, seed, 0), synth.make_params(cfg, seed, 1)
    if random_a:
        pf["A"], pb["A"] = synth.random_A(cfg, seed), synth.random_A(cfg, seed + 1)
    inp = synth.make_inputs(cfg, seed)
    inp_b = synth.make_inputs(cfg, seed + 500) if untied else None
    tol = gpu.TOL[cfg["io"]]
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), None if inp_b is None else to_np(inp_b))
    got = gpu.gpu_fwd(cfg, pf, pb, inp, inp_b)
    assert_close(got, ref, tol, (layout, cfg))
    # block entry point from a carried state and conv tail
    Bt, Dn, N, K = cfg["batch"], cfg["d_inner"], cfg["d_state"], cfg["d_conv"]
    tail_ch = Dn + (2 * cfg["n_groups"] * N if cfg["conv_bc"] else 0)
    g = torch.Generator().manual_seed(seed)
    h0 = (0.2 * torch.randn(Bt, Dn, N, generator=g)).float()
    tail0 = synth.round_io(torch.randn(Bt, K - 1, tail_ch, generator=g), cfg["io"]) if K > 1 else None
    ref, h_ref, t_ref = oracle.bimamba_block_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), None if inp_b is None else to_np(inp_b),
                                                 h_in=h0.numpy(), tail_in=None if tail0 is None else tail0.numpy())
    out, h, tail = gpu.gpu_block_fwd(cfg, pf, pb, inp, inp_b, h_in=h0, tail_in=tail0)
    assert_close(out, ref, tol, (layout, cfg))
    # the matrix-core kernels round their operands to bf16, so their committed state is looser (see the tolerances)
    P = Dn // cfg["n_heads"]
    mfma = (cfg["a_kind"] == 1 and cfg["io"] == "bf16" and N in (64, 128) and P in (32, 64)
            and cfg["time_chunks"] == 0 and cfg["state_split"] == 0)
    assert rel_l2(h, h_ref) < (1e-2 if mfma else 1e-5), (layout, cfg)
    if K > 1:
        assert np.array_equal(tail, t_ref)


@pytest.mark.parametrize("layout", ["selective", "mamba2_mfma", "mamba2_valu"])
def test_extreme_decay_and_silent_stretches(gpu, oracle, layout):
    """Steps large enough to wipe the state within one token (Delta * |A| up to ~800), steps of zero, and stretches of
    zero input: the decay factors under- and overflow only where the result is masked or multiplied by zero, so the
    output must stay finite and within tolerance."""
    if layout == "selective":
        cfg = synth.mixer_cfg(2, 200, 128, io="bf16")
    else:
        cfg = synth.m2_cfg(2, 200, 128, headdim=64, d_state=64, dt_softplus=0, state_split=0 if layout == "mamba2_mfma" else 1)
    pf, pb = synth.make_params(cfg, 77, 0), synth.make_params(cfg, 77, 1)
    inp = synth.make_inputs(cfg, 77)
    g = torch.Generator().manual_seed(78)
    scale = torch.ones(2, 200, 1)
    scale[:, 40:60] = 50.0 / 0.05          # ~50 per step
    scale[:, 120:150] = 0.0                # no step at all: the state is frozen
    inp["dt"] = synth.round_io(inp["dt"] * scale, "bf16")
    inp["x"][:, 90:110] = 0.0
    inp["x"] = synth.round_io(inp["x"] + 0.0, "bf16")
    ref = oracle.bimamba_fwd(cfg, to_np(pf), to_np(pb), to_np(inp))
    got = gpu.gpu_fwd(cfg, pf, pb, inp)
    assert np.all(np.isfinite(got))
    assert_close(got, ref, gpu.TOL["bf16"], layout)
