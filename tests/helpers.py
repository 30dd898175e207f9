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
