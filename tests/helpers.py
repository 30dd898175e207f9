"""Shared test helpers: tiny configs, numpy conversions, error metric."""
import numpy as np
import torch

from paper_2511_15927_amd import synth


def to_np(d):
    return {k: (None if v is None else v.numpy()) for k, v in d.items()}


def tiny_case(seed=1, random_a=True, **kw):
    """Small mixer case as numpy dicts: cfg, params_f, params_b, inputs."""
    base = dict(batch=2, seqlen=12, d_inner=6, d_state=4, io="f32")
    base.update(kw)
    cfg = synth.mixer_cfg(**base)
    pf = synth.make_params(cfg, seed, 0)
    pb = synth.make_params(cfg, seed, 1)
    if random_a:
        pf["A"] = synth.random_A(cfg, seed)
        pb["A"] = synth.random_A(cfg, seed + 1)
    return cfg, to_np(pf), to_np(pb), to_np(synth.make_inputs(cfg, seed))


def rel_l2(got, ref):
    """max over batch elements of ||got-ref||_2 / ||ref||_2."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    worst = 0.0
    for b in range(ref.shape[0]):
        den = np.linalg.norm(ref[b].ravel())
        num = np.linalg.norm((got[b] - ref[b]).ravel())
        if den == 0.0:
            worst = max(worst, 0.0 if num == 0.0 else np.inf)
        else:
            worst = max(worst, num / den)
    return worst


ROWWISE_FROM = 512     # sequence lengths from which the per-token bound is asserted beside the slab norm


def rowwise_rel(got, ref):
    """max over batch elements and tokens of ||got[b,t] - ref[b,t]||_2 / max(||ref[b,t]||_2, rms_t ||ref[b,t]||_2).

    One slab norm over [L, channels] hides a token row that is wrong altogether once L is a few thousand; this bound
    does not.  The floor at the root-mean-square row norm keeps rows that happen to be small from inflating it."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    Bt, L = ref.shape[0], ref.shape[1]
    if Bt == 0 or L == 0:
        return 0.0
    g, r = got.reshape(Bt, L, -1), ref.reshape(Bt, L, -1)
    worst = 0.0
    for b in range(Bt):
        rows = np.linalg.norm(r[b], axis=1)
        err = np.linalg.norm(g[b] - r[b], axis=1)
        floor = np.sqrt(np.mean(rows ** 2))
        if floor == 0.0:
            worst = max(worst, 0.0 if not err.any() else np.inf)
            continue
        worst = max(worst, float(np.max(err / np.maximum(rows, floor))))
    return worst


def assert_close(got, ref, tol, what=""):
    """The parity bar: slab relative L2 per batch element, plus, from ROWWISE_FROM tokens on, the same bound per token.
    In separate mode ([Bt, L, 2, ch]) each direction's half is held to the bound by itself."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape, what)
    halves = [(got, ref)] if ref.ndim == 3 else [(got[:, :, s], ref[:, :, s]) for s in range(ref.shape[2])]
    worst = 0.0
    for g, r in halves:
        e = rel_l2(g, r)
        assert e < tol, ("slab", e, tol, what)
        worst = max(worst, e)
        if r.shape[1] >= ROWWISE_FROM:
            ew = rowwise_rel(g, r)
            assert ew < tol, ("row-wise", ew, tol, what)
    return worst


def _kept_heads(cfg, channels):
    ch = np.asarray(channels, dtype=np.int64)
    P = cfg["d_inner"] // cfg["n_heads"]
    assert cfg["n_groups"] == 1
    if P == 1:
        return ch, ch
    assert len(ch) % P == 0 and np.array_equal(ch.reshape(-1, P), ch.reshape(-1, P)[:, :1] + np.arange(P)), "whole heads"
    return ch, ch.reshape(-1, P)[:, 0] // P


def slice_cfg(cfg, channels):
    ch, heads = _kept_heads(cfg, channels)
    return dict(cfg, d_inner=len(ch), n_heads=len(heads))


def slice_params(cfg, p, channels):
    """One direction's parameters (numpy) restricted to some channels, see slice_channels."""
    ch, heads = _kept_heads(cfg, channels)
    GN = cfg["n_groups"] * cfg["d_state"]
    rows = ch if not cfg["conv_bc"] else np.concatenate([ch, np.arange(cfg["d_inner"], cfg["d_inner"] + 2 * GN)])
    return dict(conv_w=p["conv_w"][rows], conv_b=None if p["conv_b"] is None else p["conv_b"][rows],
                A=p["A"][heads], D=p["D"][heads if cfg["d_kind"] == 1 else ch],
                dt_bias=None if p.get("dt_bias") is None else p["dt_bias"][heads])


def slice_inputs(cfg, i, channels):
    ch, heads = _kept_heads(cfg, channels)
    return dict(x=i["x"][:, :, ch], z=i["z"][:, :, ch], dt=i["dt"][:, :, heads], B=i["B"], C=i["C"])


def slice_channels(cfg, pf, pb, inp, channels):
    """The same problem restricted to some channels (numpy in, numpy out), for an oracle run that never holds the full
    tensors: every chain depends only on its own channel's x, z, D, conv taps and on its head's dt, A, dt_bias, plus the
    B and C rows, so the restriction is exact.  `channels` is a sorted list; with several channels per head it must hold
    whole heads.  Returns (cfg, pf, pb, inp) of the reduced width."""
    return (slice_cfg(cfg, channels), slice_params(cfg, pf, channels), slice_params(cfg, pb, channels),
            slice_inputs(cfg, inp, channels))


def slice_tail(cfg, tail, channels):
    """Rows of a cached conv tail [Bt, K-1, tail_ch] that belong to the channels kept by slice_channels."""
    ch = np.asarray(channels, dtype=np.int64)
    Dn = cfg["d_inner"]
    GN = cfg["n_groups"] * cfg["d_state"]
    cols = ch if not cfg["conv_bc"] else np.concatenate([ch, np.arange(Dn, Dn + 2 * GN)])
    return np.asarray(tail)[:, :, cols]
