"""Timing report over all benchmark configurations (tokens/s, algorithmic GB/s, fraction of HBM peak).

    python -m paper_2511_15927_amd.report --out report.json [--quick]

Timing only: inputs are drawn on the GPU with the recipe's distributions (parity of every configuration is the
tests' job).  Covers the 1.3B-scale layer, the long sequence, the headline shape at batch 1 and 8 with structured and
general A, the Mamba-2 parameterisation, the block-diffusion loop (prefix once, then 32-token blocks re-scanned 8
times from the cached state, eagerly and as a replayed HIP graph; then a 24-layer stack per denoising step at block
lengths 32, 64 and 128, both parameterisations) and the 24-layer batch x length sweep.
"""
import argparse
import json
import math
import sys

import torch

from . import binding as bd
from . import shapes, synth

PEAK_HBM_GBPS = 8000.0


def gpu_inputs(cfg, seed=1):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    Bt, L, Dn, H, GN = cfg["batch"], cfg["seqlen"], cfg["d_inner"], cfg["n_heads"], cfg["n_groups"] * cfg["d_state"]
    io = bd.io_dtype(cfg)
    rn = lambda *s: torch.randn(*s, device="cuda", generator=g)
    shift = synth.dt_shift(cfg, seed).cuda()
    raw = 0.5 * rn(Bt, L, H)
    dt = raw if cfg["dt_softplus"] else torch.nn.functional.softplus(raw + shift)
    return dict(x=rn(Bt, L, Dn).to(io), z=rn(Bt, L, Dn).to(io), dt=dt.to(io), B=rn(Bt, L, GN).to(io), C=rn(Bt, L, GN).to(io))


def gpu_params(cfg, seed=1, general_a=False):
    pf, pb = synth.make_params(cfg, seed, 0), synth.make_params(cfg, seed, 1)
    if general_a:
        pf["A"], pb["A"] = synth.random_A(cfg, seed), synth.random_A(cfg, seed + 1)
    return bd.to_device(pf), bd.to_device(pb)


def timed(fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_fwd(name, cfg, steps=10, warmup=3, general_a=False, untied=False):
    desc = bd.make_desc(cfg)
    dpf, dpb = gpu_params(cfg, general_a=general_a)
    inp = gpu_inputs(cfg)
    inp_b = gpu_inputs(cfg, seed=2) if untied else None   # untied directions: the reverse layer has its own x, z, dt, B, C
    out, ws = bd.alloc_out(cfg), bd.alloc_workspace(desc)
    args = (desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(inp),
            None if inp_b is None else bd.make_inputs(inp_b), bd.make_tensor(out), ws)
    ms = timed(lambda: bd.bimamba_fwd(*args), steps, warmup)
    tokens = cfg["batch"] * cfg["seqlen"]
    gbps = shapes.algorithmic_bytes(cfg, shared_inputs=not untied) / (ms * 1e-3) / 1e9
    row = dict(name=name, batch=cfg["batch"], seq_len=cfg["seqlen"], d_inner=cfg["d_inner"], d_state=cfg["d_state"],
               layout="mamba2" if cfg["a_kind"] == 1 else "selective", io=cfg["io"], A="general" if general_a else "recipe",
               inputs="per direction" if untied else "shared", combine="separate" if cfg["combine"] == 1 else "add",
               time_chunks=bd.bimamba_time_chunks(desc), ms=ms, tokens_per_s=tokens / (ms * 1e-3),
               algorithmic_GBps=gbps, hbm_frac=gbps / PEAK_HBM_GBPS,
               alu_TFLOPs=shapes.algorithmic_flops(cfg) / (ms * 1e-3) / 1e12)
    print(json.dumps(row), flush=True)
    return row


def time_block_loop(n_blocks=8, steps_per_block=8, prefix=4096):
    """Block diffusion at batch 16, d_inner 4096: prefix scanned once, then blocks of 32 tokens, each re-scanned
    `steps_per_block` times from the cached state, committing state and conv tail on a block's last step."""
    cfg_p, cfg_b = dict(synth.CONFIGS["cfg3_prefix"], seqlen=prefix), dict(synth.CONFIGS["cfg3_block"])
    Bt, Dn, N, G = cfg_b["batch"], cfg_b["d_inner"], cfg_b["d_state"], cfg_b["seqlen"]
    dpf, dpb = gpu_params(cfg_b)
    pf, pb = bd.make_params(dpf), bd.make_params(dpb)
    h = torch.zeros(Bt, Dn, N, dtype=torch.float32, device="cuda")
    tail = torch.zeros(Bt, 3, Dn, dtype=torch.bfloat16, device="cuda")
    # prefix
    dp = bd.make_desc(cfg_p)
    pin = gpu_inputs(cfg_p, 2)
    pout, pws = bd.alloc_out(cfg_p), bd.alloc_workspace(dp, 1)
    p_ms = timed(lambda: bd.bimamba_block_fwd(dp, pf, pb, bd.make_inputs(pin), None, None, None, h, tail,
                                              bd.make_tensor(pout), pws), 3, 1)
    # blocks: one set of step inputs reused for every block (timing only)
    db = bd.make_desc(cfg_b)
    step_in = [gpu_inputs(cfg_b, 10 + s) for s in range(steps_per_block)]
    c_in = [bd.make_inputs(i) for i in step_in]
    out, ws = bd.alloc_out(cfg_b), bd.alloc_workspace(db, 1)
    c_out = bd.make_tensor(out)

    def one_block():
        for s in range(steps_per_block):
            last = s == steps_per_block - 1
            bd.bimamba_block_fwd(db, pf, pb, c_in[s], None, h, tail, h if last else None, tail if last else None, c_out, ws)

    eager_ms = timed(one_block, n_blocks, 2)
    graph_ms = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            one_block()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            one_block()
        graph_ms = timed(graph.replay, n_blocks, 2)
    except Exception as exc:  # graph capture is an optimisation of the loop, not part of the path
        print("graph capture skipped: %r" % (exc,), file=sys.stderr)
    calls = steps_per_block
    row = dict(name="cfg3_block_loop", batch=Bt, block=G, d_inner=Dn, steps_per_block=steps_per_block, prefix=prefix,
               prefix_ms=p_ms, prefix_tokens_per_s=Bt * prefix / (p_ms * 1e-3),
               eager_us_per_call=eager_ms * 1e3 / calls, eager_generated_tokens_per_s=Bt * G / (eager_ms * 1e-3),
               graph_us_per_call=None if graph_ms is None else graph_ms * 1e3 / calls,
               graph_generated_tokens_per_s=None if graph_ms is None else Bt * G / (graph_ms * 1e-3))
    print(json.dumps(row), flush=True)
    return row


def time_block_stack(block, layers=synth.CFG4_LAYERS, steps_per_block=8, mamba2=False, batch=16, d_inner=4096):
    """One denoising step of a `layers`-deep stack on one block: layer l's output is layer l+1's x; z, dt, B, C are
    shared; every layer has its own parameters, cached state and conv tail.  The step that ends a block commits the
    caches.  Timed eagerly and as a replayed HIP graph of a whole block (steps_per_block steps)."""
    cfg = synth.m2_cfg(batch, block, d_inner) if mamba2 else synth.mixer_cfg(batch, block, d_inner)
    desc = bd.make_desc(cfg)
    N, K = cfg["d_state"], cfg["d_conv"]
    tail_ch = d_inner + (2 * cfg["n_groups"] * N if cfg["conv_bc"] else 0)
    inp = gpu_inputs(cfg)
    params = [gpu_params(cfg, seed=200 + l) for l in range(layers)]
    cparams = [(bd.make_params(a), bd.make_params(b)) for a, b in params]
    h = [torch.zeros(batch, d_inner, N, dtype=torch.float32, device="cuda") for _ in range(layers)]
    tail = [torch.zeros(batch, K - 1, tail_ch, dtype=torch.bfloat16, device="cuda") for _ in range(layers)]
    bufs = [inp["x"], bd.alloc_out(cfg), bd.alloc_out(cfg)]
    ws = bd.alloc_workspace(desc, 1)
    c_in = [bd.make_inputs(dict(inp, x=b)) for b in bufs]
    c_out = [bd.make_tensor(b) for b in bufs]

    def one_block():
        for s in range(steps_per_block):
            last = s == steps_per_block - 1
            src = 0
            for l in range(layers):
                dst = 1 if src != 1 else 2
                bd.bimamba_block_fwd(desc, cparams[l][0], cparams[l][1], c_in[src], None, h[l], tail[l],
                                     h[l] if last else None, tail[l] if last else None, c_out[dst], ws)
                src = dst

    eager_ms = timed(one_block, 3, 1)
    graph_ms = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            one_block()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            one_block()
        graph_ms = timed(graph.replay, 3, 1)
    except Exception as exc:  # graph capture is an optimisation of the loop, not part of the path
        print("graph capture skipped: %r" % (exc,), file=sys.stderr)
    best = eager_ms if graph_ms is None else min(eager_ms, graph_ms)
    row = dict(name="block_stack", layout="mamba2" if mamba2 else "selective", batch=batch, block=block, d_inner=d_inner,
               layers=layers, steps_per_block=steps_per_block, eager_ms_per_block=eager_ms, graph_ms_per_block=graph_ms,
               us_per_layer_call=best * 1e3 / (layers * steps_per_block),
               generated_tokens_per_s=batch * block / (best * 1e-3))
    print(json.dumps(row), flush=True)
    return row


def time_stack(batch, seqlen, layers=synth.CFG4_LAYERS, steps=2):
    """24 mixer layers back to back: layer l's output is layer l+1's x; z, dt, B, C are shared by all layers;
    every layer has its own seeded parameters."""
    cfg = synth.cfg4(batch, seqlen)
    desc = bd.make_desc(cfg)
    inp = gpu_inputs(cfg)
    params = [gpu_params(cfg, seed=100 + l) for l in range(layers)]
    cparams = [(bd.make_params(a), bd.make_params(b)) for a, b in params]
    bufs = [inp["x"], bd.alloc_out(cfg), bd.alloc_out(cfg)]
    ws = bd.alloc_workspace(desc)

    def run():
        src = 0
        for l in range(layers):
            dst = 1 if src != 1 else 2
            cur = dict(inp, x=bufs[src])
            bd.bimamba_fwd(desc, cparams[l][0], cparams[l][1], bd.make_inputs(cur), None, bd.make_tensor(bufs[dst]), ws)
            src = dst

    ms = timed(run, steps, 1)
    tokens = batch * seqlen
    gbps = layers * shapes.algorithmic_bytes(cfg) / (ms * 1e-3) / 1e9
    row = dict(name="cfg4_stack", batch=batch, seq_len=seqlen, d_inner=cfg["d_inner"], layers=layers, ms=ms,
               tokens_per_s=tokens / (ms * 1e-3), token_layers_per_s=tokens * layers / (ms * 1e-3),
               algorithmic_GBps=gbps, hbm_frac=gbps / PEAK_HBM_GBPS, time_chunks=bd.bimamba_time_chunks(desc))
    print(json.dumps(row), flush=True)
    return row


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=None)
    ap.add_argument("--quick", action="store_true", help="skip the long Mamba-2 VALU runs and the largest sweep points")
    ap.add_argument("--only", default=None, help="comma-separated subset: fwd, m2, block, stack")
    a = ap.parse_args()
    want = set((a.only or "fwd,m2,block,stack").split(","))
    assert torch.cuda.is_available()
    bd.lib()
    rows = []
    C = synth.CONFIGS
    if "fwd" in want:
        rows.append(time_fwd("cfg0", C["cfg0"]))
        rows.append(time_fwd("cfg1", C["cfg1"]))
        rows.append(time_fwd("cfg2", C["cfg2"]))
        rows.append(time_fwd("headline_b8", C["headline"]))
        rows.append(time_fwd("headline_b8_generalA", C["headline"], general_a=True))
        rows.append(time_fwd("headline_b1", C["headline_b1"]))
        rows.append(time_fwd("headline_b8_shared_separate", dict(C["headline"], combine=1)))
        rows.append(time_fwd("headline_b8_untied_separate", dict(C["headline"], combine=1), untied=True))
    if "m2" in want:
        rows.append(time_fwd("cfg0_m2", C["cfg0_m2"]))
        m2 = dict(C["cfg1_m2"]) if not a.quick else dict(C["cfg1_m2"], batch=1)
        rows.append(time_fwd("cfg1_m2" if not a.quick else "cfg1_m2_batch1", m2, steps=2, warmup=1))
        if not a.quick:
            rows.append(time_fwd("headline_m2_b8", synth.m2_cfg(8, 8192, 4096), steps=2, warmup=1))
            rows.append(time_fwd("paper_1p3b_layer_b8_L8192", synth.m2_cfg(8, 8192, 3840, headdim=32), steps=2, warmup=1))
    if "block" in want:
        rows.append(time_block_loop())
        for block in (32, 64, 128):
            rows.append(time_block_stack(block))
            rows.append(time_block_stack(block, mamba2=True))
    if "stack" in want:
        for bt in synth.CFG4_BATCHES:
            for L in synth.CFG4_LENGTHS:
                if a.quick and bt * L > 8 * 8192:
                    continue
                rows.append(time_stack(bt, L))
    if a.out:
        with open(a.out, "w") as f:
            json.dump(rows, f, indent=1)


if __name__ == "__main__":
    main()
