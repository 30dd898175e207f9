"""GPU parity of bimamba_bwd (gradients of the full-sequence path, selective-scan layout) against the fp64 oracle's
gradients, which are themselves pinned by finite differences and automatic differentiation (test_oracle_bwd_pins.py).

Tolerances: a gradient tensor is compared in relative L2 over the whole tensor; fp32 I/O 2e-5 (fp32 arithmetic, sums of
up to L * batch terms formed with atomics in arbitrary order), bf16 I/O 2e-2 for the tensors that are rounded to bf16
(dx, dz, ddt) and 2e-5 for the fp32 ones (dB, dC and the parameter gradients see the same fp32 arithmetic in both modes).
"""
import numpy as np
import pytest
import torch

from helpers import rel_l2, to_np
from paper_2511_15927_amd import binding as bd
from paper_2511_15927_amd import synth
from test_gpu_block import params

pytestmark = pytest.mark.gpu

FP32_TOL, BF16_TOL = 2e-5, 2e-2


@pytest.fixture(scope="module")
def gpu():
    import gpu_util
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return gpu_util


def rounded(a, io):
    t = torch.as_tensor(a, dtype=torch.float32)
    return (t.to(torch.bfloat16).float() if io == "bf16" else t).numpy()


def rel_all(got, ref):
    """Relative L2 over a whole tensor (parameter gradients have no batch dimension to take a maximum over)."""
    return float(np.linalg.norm(np.asarray(got) - np.asarray(ref)) / np.linalg.norm(np.asarray(ref)))


def compare(cfg, got, ref, sel=None):
    io_tol = BF16_TOL if cfg["io"] == "bf16" else FP32_TOL
    gf, gb, qf, qb = got
    rf, rb, pf, pb = ref
    pick = (lambda a: a[..., sel]) if sel is not None else (lambda a: a)
    worst = {}
    for tag, g, r in (("f", gf, rf), ("b", gb, rb)):
        if r is None:
            assert g is None
            continue
        for k in ("dx", "dz"):
            worst[tag + k] = rel_l2(pick(g[k]), r[k])
            assert worst[tag + k] < io_tol, (tag, k, worst)
        worst[tag + "ddt"] = rel_l2(pick(g["ddt"]), pick(r["ddt"]))
        assert worst[tag + "ddt"] < io_tol, (tag, "ddt", worst)
        if sel is None:
            for k in ("dB", "dC"):
                worst[tag + k] = rel_l2(g[k], r[k])
                assert worst[tag + k] < FP32_TOL, (tag, k, worst)
    for tag, g, r in (("f", qf, pf), ("b", qb, pb)):
        for k in ("dconv_w", "dconv_b", "dA", "dD", "ddt_bias"):
            a, b = (g[k][sel], r[k][sel]) if sel is not None else (g[k], r[k])
            if not np.any(b):
                assert not np.any(a), (tag, k)
                continue
            worst[tag + k] = rel_all(a, b)
            assert worst[tag + k] < FP32_TOL, (tag, k, worst)
    return worst


def run_case(gpu, oracle, cfg, seed, untied=False, random_a=True):
    pf, pb = params(cfg, seed, random_a=random_a)
    in_f = synth.make_inputs(cfg, seed)
    in_b = synth.make_inputs(cfg, seed + 500) if untied else None
    width = cfg["d_inner"] * (2 if cfg["combine"] else 1)
    g = torch.Generator().manual_seed(seed + 9)
    dout = rounded(torch.randn(cfg["batch"], cfg["seqlen"], width, generator=g), cfg["io"])
    got = gpu.gpu_bwd(cfg, pf, pb, in_f, in_b, dout)
    ref = oracle.bimamba_bwd(cfg, to_np(pf), to_np(pb), to_np(in_f), None if in_b is None else to_np(in_b), dout)
    return compare(cfg, got, ref)


@pytest.mark.parametrize("L", [1, 2, 7, 8, 9, 16, 23, 100])
@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_lengths_around_the_chunks(gpu, oracle, L, io):
    run_case(gpu, oracle, synth.mixer_cfg(2, L, 72, io=io), 10 + L)


@pytest.mark.parametrize("N", [4, 8, 16])
@pytest.mark.parametrize("K", [1, 2, 3, 4])
def test_state_sizes_and_conv_widths(gpu, oracle, N, K):
    run_case(gpu, oracle, synth.mixer_cfg(2, 37, 130, d_state=N, d_conv=K, io="f32"), 30 + N + K)


@pytest.mark.parametrize("mode", ["separate", "untied", "untied_separate", "softplus", "groups", "progression_a"])
def test_modes(gpu, oracle, mode):
    kw = {}
    if "separate" in mode:
        kw["combine"] = synth.COMBINE_SEPARATE
    if mode == "softplus":
        kw["dt_softplus"] = 1
    Dn = 256 if mode == "groups" else 96
    if mode == "groups":
        kw["n_groups"] = 2
    cfg = synth.mixer_cfg(3, 45, Dn, io="f32", **kw)
    run_case(gpu, oracle, cfg, 77, untied="untied" in mode, random_a=mode != "progression_a")


@pytest.mark.parametrize("seed", range(32))
def test_random_descriptor(gpu, oracle, seed):
    """Seeded random draws from the supported space: state count, conv width, length (around the chunks of 8 or 16 and
    the meeting point of the two walks), channel counts with ragged tiles and shadow waves, groups, modes, dtypes."""
    rng = np.random.default_rng(4100 + seed)
    N = int(rng.choice([4, 8, 16]))
    G = int(rng.choice([1, 1, 2]))
    Dn = int(rng.choice([128, 256, 384])) if G == 2 else int(rng.choice([1, 7, 64, 100, 130, 192, 200]))
    L = int(rng.choice([1, 2, 3, 5, 15, 17, 31, 33, 48, 65, 97]))
    cfg = synth.mixer_cfg(int(rng.integers(1, 4)), L, Dn, d_state=N, d_conv=int(rng.integers(1, 5)), n_groups=G,
                          io=str(rng.choice(["f32", "bf16"])), combine=int(rng.integers(0, 2)),
                          dt_softplus=int(rng.integers(0, 2)))
    run_case(gpu, oracle, cfg, 600 + seed, untied=bool(rng.integers(0, 2)), random_a=bool(rng.integers(0, 2)))


def test_gradient_call_replayed_from_a_hip_graph(gpu):
    """bimamba_bwd captured into a HIP graph (it clears its accumulation targets with kernels, not memset nodes):
    every replay, with eager work and synchronisation between replays and fresh contents in the static buffers, must
    equal the eager call on the same contents: bit for bit for the activation gradients (fixed summation order), to
    rounding for the parameter gradients (their sum over the batch is formed with atomics)."""
    cfg = synth.mixer_cfg(3, 45, 200, io="bf16")
    Bt, L, Dn, N, K = 3, 45, 200, cfg["d_state"], cfg["d_conv"]
    pf, pb = params(cfg, 5)
    dpf, dpb = bd.to_device(pf), bd.to_device(pb)
    desc = bd.make_desc(cfg)
    static_in = bd.to_device(synth.make_inputs(cfg, 5), cfg)
    dout = torch.zeros(Bt, L, Dn, dtype=torch.bfloat16, device="cuda")
    io = torch.bfloat16
    gi = dict(dx=torch.empty(Bt, L, Dn, dtype=io, device="cuda"), dz=torch.empty(Bt, L, Dn, dtype=io, device="cuda"),
              ddt=torch.empty(Bt, L, Dn, dtype=io, device="cuda"), dB=torch.empty(Bt, L, 1, N, device="cuda"),
              dC=torch.empty(Bt, L, 1, N, device="cuda"))
    mk = lambda: dict(dconv_w=torch.empty(Dn, K, device="cuda"), dconv_b=torch.empty(Dn, device="cuda"),
                      dA=torch.empty(Dn, N, device="cuda"), dD=torch.empty(Dn, device="cuda"), ddt_bias=torch.empty(Dn, device="cuda"))
    qf, qb = mk(), mk()
    ws = torch.empty(bd.bimamba_bwd_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    args = (desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(static_in), None, bd.make_tensor(dout),
            bd.make_input_grads(gi), None, bd.make_param_grads(qf), bd.make_param_grads(qb), ws)

    def call():
        bd.bimamba_bwd(*args)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    outs = list(gi.values()) + list(qf.values()) + list(qb.values())
    n_exact = len(gi)
    for rep in range(3):
        fresh = bd.to_device(synth.make_inputs(cfg, 70 + rep), cfg)
        for k in static_in:
            static_in[k].copy_(fresh[k])
        dout.copy_(torch.randn(Bt, L, Dn, generator=torch.Generator().manual_seed(80 + rep)).to(io))
        call()
        torch.cuda.synchronize()
        want = [t.clone() for t in outs]
        for t in outs:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, ref) in enumerate(zip(outs, want)):
            if i < n_exact:
                assert torch.equal(got, ref), (rep, i)
            elif not bool(ref.any()):
                assert not bool(got.any()), (rep, i)      # e.g. the Delta bias without softplus
            else:
                assert rel_all(got.cpu().numpy(), ref.cpu().numpy()) < 1e-6, (rep, i)


@pytest.mark.parametrize("untied", [False, True])
def test_column_slices_with_their_own_token_strides(gpu, oracle, untied):
    """x, z, dt as column slices of one wide buffer per direction, dout a slice of another, dx, dz, ddt slices of a
    third: every tensor has its own row pitch, and the kernels step through each with its own stride.  Nothing outside
    the gradient views may be written."""
    cfg = synth.mixer_cfg(2, 37, 72, io="bf16", combine=synth.COMBINE_SEPARATE)
    Bt, L, Dn, N, K = 2, 37, 72, cfg["d_state"], cfg["d_conv"]
    io = torch.bfloat16
    pf, pb = params(cfg, 3)
    ins = [synth.make_inputs(cfg, 3)] + ([synth.make_inputs(cfg, 503)] if untied else [])
    g = torch.Generator().manual_seed(12)
    dout = rounded(torch.randn(Bt, L, 2 * Dn, generator=g), "bf16")

    def sliced(t, width, at):
        wide = torch.zeros(Bt, L, width, dtype=io, device="cuda")
        view = wide[..., at:at + t.shape[-1]]
        view.copy_(torch.as_tensor(t).to(io))
        return wide, view

    dev_in, grads, wides = [], [], []
    for inp in ins:
        d = bd.to_device(inp, cfg)
        d["x"] = sliced(inp["x"], 3 * Dn + 40, 8)[1]
        d["z"] = sliced(inp["z"], 2 * Dn + 24, 16)[1]
        d["dt"] = sliced(inp["dt"], Dn + 8, 0)[1]
        dev_in.append(d)
        wide = torch.zeros(Bt, L, 3 * Dn + 48, dtype=io, device="cuda")
        wides.append(wide)
        grads.append(dict(dx=wide[..., 8:8 + Dn], dz=wide[..., 16 + Dn:16 + 2 * Dn], ddt=wide[..., 40 + 2 * Dn:40 + 3 * Dn],
                          dB=torch.empty(Bt, L, 1, N, device="cuda"), dC=torch.empty(Bt, L, 1, N, device="cuda")))
    do = sliced(dout, 2 * Dn + 64, 32)[1]
    mk = lambda: dict(dconv_w=torch.empty(Dn, K, device="cuda"), dconv_b=torch.empty(Dn, device="cuda"),
                      dA=torch.empty(Dn, N, device="cuda"), dD=torch.empty(Dn, device="cuda"), ddt_bias=torch.empty(Dn, device="cuda"))
    qf, qb = mk(), mk()
    desc = bd.make_desc(cfg)
    dpf, dpb = bd.to_device(pf), bd.to_device(pb)
    ws = torch.empty(bd.bimamba_bwd_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    bd.bimamba_bwd(desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(dev_in[0]),
                   bd.make_inputs(dev_in[1]) if untied else None, bd.make_tensor(do), bd.make_input_grads(grads[0]),
                   bd.make_input_grads(grads[1]) if untied else None, bd.make_param_grads(qf), bd.make_param_grads(qb), ws)
    torch.cuda.synchronize()
    host = lambda d: {k: v.float().cpu().numpy().astype(np.float64) for k, v in d.items()}
    got = (host(grads[0]), host(grads[1]) if untied else None, host(qf), host(qb))
    ref = oracle.bimamba_bwd(cfg, to_np(pf), to_np(pb), to_np(ins[0]), to_np(ins[1]) if untied else None, dout)
    compare(cfg, got, ref)
    for wide in wides:
        for lo, hi in ((0, 8), (8 + Dn, 16 + Dn), (16 + 2 * Dn, 40 + 2 * Dn), (40 + 3 * Dn, 48 + 3 * Dn)):
            assert float(wide[..., lo:hi].abs().max()) == 0.0


@pytest.mark.parametrize("N", [4, 8, 16])
@pytest.mark.parametrize("L", [1, 5, 37, 70])
def test_more_waves_than_simds_takes_the_dense_form(gpu, oracle, N, L):
    """Batch 9 at d_inner 4096 is 1152 waves for 1024 SIMDs: the kernels built for two waves per SIMD (shorter chunks
    for 4 and 16 states) and the plan that sizes their stored states; every channel compared."""
    run_case(gpu, oracle, synth.mixer_cfg(9, L, 4096, d_state=N, io="bf16" if L % 2 else "f32"), 900 + N + L)


def test_empty_call_zeroes_the_parameter_gradients(gpu, oracle):
    cfg = synth.mixer_cfg(0, 16, 64, io="f32")
    pf, pb = params(cfg, 1)
    got = gpu.gpu_bwd(cfg, pf, pb, synth.make_inputs(cfg, 1), None, np.zeros((0, 16, 64), dtype=np.float32))
    assert got[0]["dx"].shape == (0, 16, 64)
    for q in got[2:]:
        assert all(not np.any(v) for v in q.values())


def test_unsupported_layouts_are_refused_on_the_host(gpu):
    for cfg in (synth.m2_cfg(1, 64, 128, headdim=64, d_state=64), synth.mixer_cfg(1, 8, 64, d_state=32)):
        assert bd.bimamba_bwd_workspace_bytes(bd.make_desc(cfg)) == 0


def test_headline_width_sampled(gpu, oracle):
    """d_inner 4096, bf16, a few hundred tokens: the x / z / Delta and per-channel parameter gradients on sampled
    channels (B and C gradients are sums over all channels and are covered by the small cases)."""
    cfg = synth.mixer_cfg(2, 300, 4096)
    pf, pb = params(cfg, 5, random_a=False)
    inp = synth.make_inputs(cfg, 5)
    g = torch.Generator().manual_seed(3)
    dout = rounded(torch.randn(2, 300, 4096, generator=g), "bf16")
    sel = list(range(3, 4096, 511))
    got = gpu.gpu_bwd(cfg, pf, pb, inp, None, dout)
    ref = oracle.bimamba_bwd(cfg, to_np(pf), to_np(pb), to_np(inp), None, dout[..., sel], sel=sel)
    compare(cfg, got, ref, sel=sel)
