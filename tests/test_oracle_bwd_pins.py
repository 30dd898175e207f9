"""Pins of the oracle's gradients (oracle.bimamba_bwd) to things other than itself.

1. Central finite differences of the oracle's own forward, Richardson-extrapolated (error O(h^4)), for EVERY element of
   every input and parameter on small shapes: the loss is sum(R * out) with a fixed random R, so dout = R.  Inputs are
   snapped to multiples of 2^-10 so that x +- h and x +- h/2 are exact in float32 (the oracle takes float32 arrays).
2. Automatic differentiation: the forward definition written with torch's differentiable float64 ops (a python loop
   over tokens), gradients by torch.autograd, for both parameterisations.
A dropped term, a wrong sign, an off-by-one in the conv window or in which state (before / after the step) a product
uses, or a transposed B / C fails both.
"""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2511_15927_amd import synth

H1 = 2.0 ** -6


def snap(a):
    return (np.round(np.asarray(a, dtype=np.float64) * 1024.0) / 1024.0).astype(np.float32)


def make_case(cfg, seed):
    to = lambda d: {k: (None if v is None else snap(v.numpy())) for k, v in d.items()}
    pf, pb = to(synth.make_params(cfg, seed, 0)), to(synth.make_params(cfg, seed, 1))
    pf["A"], pb["A"] = snap(synth.random_A(cfg, seed).numpy()), snap(synth.random_A(cfg, seed + 1).numpy())
    inp = to(synth.make_inputs(cfg, seed))
    inp["dt"] = snap(np.abs(inp["dt"]) + 0.0625) if not cfg["dt_softplus"] else inp["dt"]
    return pf, pb, inp


def loss(cfg, pf, pb, in_f, in_b, R):
    return float((orc.bimamba_fwd(cfg, pf, pb, in_f, in_b) * R).sum())


def fd_grad(f, arr):
    """d f / d arr by Richardson-extrapolated central differences with steps H1 and H1/2 (both exact in float32)."""
    g = np.zeros(arr.shape, dtype=np.float64)
    flat = arr.reshape(-1)
    for i in range(flat.size):
        keep = flat[i]
        vals = {}
        for h in (H1, H1 / 2):
            flat[i] = keep + np.float32(h)
            up = f()
            flat[i] = keep - np.float32(h)
            dn = f()
            vals[h] = (up - dn) / (2 * h)
        flat[i] = keep
        g.reshape(-1)[i] = (4.0 * vals[H1 / 2] - vals[H1]) / 3.0
    return g


CASES = {
    "selective": synth.mixer_cfg(2, 7, 3, d_state=4, io="f32"),
    "selective_softplus_k2": synth.mixer_cfg(1, 6, 2, d_state=4, io="f32", dt_softplus=1, d_conv=2),
    "separate": synth.mixer_cfg(1, 5, 2, d_state=4, io="f32", combine=synth.COMBINE_SEPARATE),
    "grouped_heads": synth.mixer_cfg(1, 5, 4, d_state=4, n_heads=2, n_groups=2, a_kind=synth.A_SCALAR_PER_HEAD,
                                     d_kind=synth.D_PER_HEAD, dt_softplus=1, io="f32"),
    "mamba2_conv_bc": synth.m2_cfg(1, 6, 4, headdim=2, d_state=4, io="f32"),
}


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("untied", [False, True])
def test_gradients_equal_finite_differences_of_the_forward(name, untied):
    cfg = CASES[name]
    pf, pb, in_f = make_case(cfg, 5)
    in_b = make_case(cfg, 6)[2] if untied else None
    rng = np.random.default_rng(3)
    out_shape = orc.bimamba_fwd(cfg, pf, pb, in_f, in_b).shape
    R = rng.standard_normal(out_shape)
    gf, gb, qf, qb = orc.bimamba_bwd(cfg, pf, pb, in_f, in_b, R)
    f = lambda: loss(cfg, pf, pb, in_f, in_b, R)
    scale = max(1.0, float(np.abs(R).max()))
    for key, got in (("x", gf["dx"]), ("z", gf["dz"]), ("dt", gf["ddt"]), ("B", gf["dB"]), ("C", gf["dC"])):
        ref = fd_grad(f, in_f[key])
        assert np.allclose(got.reshape(ref.shape), ref, rtol=2e-5, atol=2e-6 * scale), (name, key)
    if untied:
        for key, got in (("x", gb["dx"]), ("z", gb["dz"]), ("dt", gb["ddt"]), ("B", gb["dB"]), ("C", gb["dC"])):
            ref = fd_grad(f, in_b[key])
            assert np.allclose(got.reshape(ref.shape), ref, rtol=2e-5, atol=2e-6 * scale), (name, "b", key)
    for p, q, tag in ((pf, qf, "f"), (pb, qb, "b")):
        for key, gkey in (("conv_w", "dconv_w"), ("conv_b", "dconv_b"), ("A", "dA"), ("D", "dD"), ("dt_bias", "ddt_bias")):
            if p.get(key) is None or (key == "dt_bias" and not cfg["dt_softplus"]):
                continue
            ref = fd_grad(f, p[key])
            assert np.allclose(q[gkey].reshape(ref.shape), ref, rtol=2e-5, atol=2e-6 * scale), (name, tag, key)


def torch_forward(cfg, p, i, direction):
    """One direction of the definition with differentiable float64 tensor ops: g [batch, L, d_inner]."""
    Bt, L, Dn, N, H, G, K = (cfg[k] for k in ("batch", "seqlen", "d_inner", "d_state", "n_heads", "n_groups", "d_conv"))
    P, HG = Dn // H, H // G
    silu = torch.nn.functional.silu

    def conv(src, w, b):                      # src [Bt, L, C], w [C, K], b [C]
        acc = b.expand(Bt, L, -1).clone() if b is not None else torch.zeros_like(src)
        for k in range(K):
            back = K - 1 - k
            shifted = torch.zeros_like(src)
            if back == 0:
                shifted = src
            elif back < L:
                if direction > 0:
                    shifted = torch.cat([torch.zeros(Bt, back, src.shape[2], dtype=src.dtype), src[:, :L - back]], 1)
                else:
                    shifted = torch.cat([src[:, back:], torch.zeros(Bt, back, src.shape[2], dtype=src.dtype)], 1)
            acc = acc + w[:, k] * shifted
        return silu(acc)

    xc = conv(i["x"], p["conv_w"][:Dn], None if p["conv_b"] is None else p["conv_b"][:Dn])
    Bm, Cm = i["B"].reshape(Bt, L, G * N), i["C"].reshape(Bt, L, G * N)
    if cfg["conv_bc"]:
        GN = G * N
        Bm = conv(Bm, p["conv_w"][Dn:Dn + GN], None if p["conv_b"] is None else p["conv_b"][Dn:Dn + GN])
        Cm = conv(Cm, p["conv_w"][Dn + GN:], None if p["conv_b"] is None else p["conv_b"][Dn + GN:])
    Bm, Cm = Bm.reshape(Bt, L, G, N), Cm.reshape(Bt, L, G, N)
    dt = i["dt"]
    if cfg["dt_softplus"]:
        dt = torch.nn.functional.softplus(dt + (p["dt_bias"] if p["dt_bias"] is not None else 0.0))
    delta = dt.repeat_interleave(P, dim=2)                                   # [Bt, L, Dn]
    A = p["A"] if cfg["a_kind"] == 0 else p["A"][:, None].expand(H, N)
    A = A.repeat_interleave(P, dim=0)                                        # [Dn, N]
    Dv = p["D"] if cfg["d_kind"] == 0 else p["D"].repeat_interleave(P)
    grp = torch.arange(Dn) // P // HG
    h = torch.zeros(Bt, Dn, N, dtype=torch.float64)
    ys = [None] * L
    order = range(L) if direction > 0 else range(L - 1, -1, -1)
    for t in order:
        Bt_, Ct_ = Bm[:, t][:, grp], Cm[:, t][:, grp]                        # [Bt, Dn, N]
        h = torch.exp(delta[:, t, :, None] * A) * h + delta[:, t, :, None] * Bt_ * xc[:, t, :, None]
        ys[t] = (Ct_ * h).sum(-1) + Dv * xc[:, t]
    return torch.stack(ys, 1) * silu(i["z"])


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("untied", [False, True])
def test_gradients_equal_automatic_differentiation(name, untied):
    cfg = dict(CASES[name], seqlen=9, batch=2)
    pf, pb, in_f = make_case(cfg, 11)
    in_b = make_case(cfg, 12)[2] if untied else None
    leaf = lambda d: {k: (None if v is None else torch.tensor(np.asarray(v, dtype=np.float64), requires_grad=True))
                      for k, v in d.items()}
    tpf, tpb, tif = leaf(pf), leaf(pb), leaf(in_f)
    tib = leaf(in_b) if untied else tif
    g_f, g_b = torch_forward(cfg, tpf, tif, +1), torch_forward(cfg, tpb, tib, -1)
    out = g_f + g_b if cfg["combine"] == 0 else torch.stack([g_f, g_b], 2)
    ref_out = orc.bimamba_fwd(cfg, pf, pb, in_f, in_b)
    assert np.allclose(out.detach().numpy(), ref_out, rtol=1e-12, atol=1e-12)      # the two forwards are the same function
    R = np.random.default_rng(8).standard_normal(ref_out.shape)
    (out * torch.tensor(R)).sum().backward()
    gf, gb, qf, qb = orc.bimamba_bwd(cfg, pf, pb, in_f, in_b, R)
    close = lambda a, t: np.allclose(a.reshape(t.shape), t.grad.numpy(), rtol=1e-10, atol=1e-11)
    for key, gk in (("x", "dx"), ("z", "dz"), ("dt", "ddt"), ("B", "dB"), ("C", "dC")):
        assert close(gf[gk], tif[key]), (name, key)
        if untied:
            assert close(gb[gk], tib[key]), (name, "b", key)
    for tp, q, tag in ((tpf, qf, "f"), (tpb, qb, "b")):
        for key, gk in (("conv_w", "dconv_w"), ("conv_b", "dconv_b"), ("A", "dA"), ("D", "dD"), ("dt_bias", "ddt_bias")):
            if tp.get(key) is None or tp[key].grad is None:
                continue
            assert close(q[gk], tp[key]), (name, tag, key)


def test_channel_selection_matches_the_full_result():
    cfg = synth.mixer_cfg(2, 11, 6, d_state=4, io="f32")
    pf, pb, inp = make_case(cfg, 2)
    R = np.random.default_rng(1).standard_normal((2, 11, 6))
    gf, _, qf, qb = orc.bimamba_bwd(cfg, pf, pb, inp, None, R)
    sel = [1, 4]
    sf, _, sqf, sqb = orc.bimamba_bwd(cfg, pf, pb, inp, None, R[..., sel], sel=sel)
    assert np.array_equal(sf["dx"], gf["dx"][..., sel]) and np.array_equal(sf["dz"], gf["dz"][..., sel])
    assert np.array_equal(sf["ddt"][..., sel], gf["ddt"][..., sel])
    assert np.array_equal(sqf["dA"][sel], qf["dA"][sel]) and np.array_equal(sqb["dconv_w"][sel], qb["dconv_w"][sel])
