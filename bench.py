#!/usr/bin/env python3
"""Benchmark of the bidirectional Mamba mixer path on one MI355X.

A step is one bimamba_fwd call (B|C preparation + bidirectional scan + gate + combine) over one batch of synthetic
input already resident in HBM.  Prints ONE JSON line: whole-job tokens/s, the roofline of the dominant kernel
(timed with HIP events around that kernel inside the timed region) and the fp64 oracle timed on the host cores on a
bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0          # MI355X HBM3E
PEAK_FP32_UNPACKED_TFLOPS = 256 * 4 * 16 * 2 * 2.4e9 / 1e12   # 78.6: one fp32 FMA per lane and clock
PEAK_FP32_VECTOR_TFLOPS = 157.3  # MI355X fp32 vector (256 CUs x 2.4 GHz x 256 flop/clk)
PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16 matrix


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200,
                    help="timed steps; the chip takes a few milliseconds of continuous work to reach its sustained rate, so "
                         "short runs read 2-8 %% low")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--probe-every", type=int, default=8, help="HIP-event pair around the dominant kernel on every n-th timed step")
    ap.add_argument("--workload", default="headline", help="name in synth.CONFIGS (default: d_inner=4096, L=8192, batch 8, bf16)")
    ap.add_argument("--general-a", action="store_true", help="draw A with no structure across states")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-general-a", action="store_true",
                    help="skip the structure-free-A comparison leg (profiling runs: it launches the same kernel)")
    ap.add_argument("--cpu-batches", type=int, default=2, help="batch elements the oracle is timed on")
    ap.add_argument("--layers", type=int, default=24, help="cfg3_block*: mixer layers in the decode loop")
    ap.add_argument("--denoise-steps", type=int, default=8, help="cfg3_block*: denoising steps per block")
    ap.add_argument("--block", type=int, default=32, help="cfg3_block*: block length G (32, 64 or 128)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run three 1 GiB device-to-device copies (a known-size reference for HBM counters)")
    return ap.parse_args()


def read_profile(kernel_key):
    """The committed rocprofv3 --pmc summary of this workload's dominant kernel (profiles/<key>_pmc.txt, written by
    paper_2511_15927_amd.profile_summary): counters as floats, plus the kernel name and the file the values come from.
    These are STORED values of an earlier run of this same command, not measurements of the present run."""
    path = os.path.join(ROOT, "profiles", kernel_key + "_pmc.txt")
    sections, kernel, shared = {}, None, {}
    try:
        for line in open(path):
            if line.startswith("# kernel:"):
                kernel = line.split(":", 1)[1].strip()
                sections[kernel] = {}
            elif "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                (sections[kernel] if kernel else shared)[k.strip()] = float(v.strip())
    except Exception:
        return {}, None, None
    ours = {k: v for k, v in sections.items() if "bm::" in k}
    if not ours:
        return {}, None, None
    # the dominant kernel of the step: the one with the longest dispatch
    kernel = max(ours, key=lambda k: ours[k].get("DURATION_NS_UNDER_PMC", 0.0))
    return dict(shared, **ours[kernel]), kernel, os.path.relpath(path, ROOT)


def traffic_of(c, launches):
    """HBM bytes per step of the dominant kernel (fetch + write, each scaled by the copy calibration)."""
    try:
        return launches * (c["FETCH_BYTES_PER_LAUNCH"] + c["WRITE_BYTES_PER_LAUNCH"])
    except KeyError:
        return None


def valu_busy_of(c, simds):
    """Fraction of SIMD time with a vector-ALU instruction executing, from the stored counters: VALU-active wave cycles
    (counted in units of four cycles) over SIMDs x the dispatch's duration at the nominal 2.4 GHz clock.  Also the
    time-averaged number of waves resident per SIMD (wave cycles over the same denominator)."""
    try:
        denom = simds * c["DURATION_NS_UNDER_PMC"] * 2.4
        return min(1.0, 4.0 * c["SQ_ACTIVE_INST_VALU"] / denom), 4.0 * c["SQ_WAVE_CYCLES"] / denom
    except (KeyError, ZeroDivisionError):
        return None, None


SHADER_ENGINES = 32   # SQ_BUSY_CYCLES is summed over the shader engines (8 XCDs x 4)


def sustained_clock_of(c, simds):
    """The shader clock the dispatch actually ran at under the counters (busy cycles of one shader engine over the
    dispatch's duration), and the vector-ALU busy fraction in those cycles rather than at the nominal clock."""
    try:
        cycles = c["SQ_BUSY_CYCLES"] / SHADER_ENGINES
        return cycles / c["DURATION_NS_UNDER_PMC"], min(1.0, 4.0 * c["SQ_ACTIVE_INST_VALU"] / (simds * cycles))
    except (KeyError, ZeroDivisionError):
        return None, None


def copy_ceiling_gbps(torch):
    """Read + write rate of a plain 1 GiB device-to-device copy, measured now (the achievable HBM ceiling on this machine)."""
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return 5 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9


def decode_loop_bench(args, torch, bd, shapes, synth):
    """Block-diffusion decode loop (Sec. 4.3): one step of this benchmark is one block of G tokens taken through
    --denoise-steps steps x --layers mixer layers (that many bimamba_block_fwd calls, the last step committing every
    layer's cache), replayed from a HIP graph captured once."""
    from paper_2511_15927_amd.decode import BlockDecodeLoop
    cfg = dict(synth.CONFIGS[args.workload], seqlen=args.block)
    seed = synth.config_seed(3)
    params = [(synth.make_params(cfg, seed + l, 0), synth.make_params(cfg, seed + l, 1)) for l in range(args.layers)]
    loop = BlockDecodeLoop(cfg, params, args.denoise_steps)
    for s in range(args.denoise_steps):
        loop.set_step_inputs(s, synth.make_inputs(cfg, seed + 100 + s))
    g = torch.Generator().manual_seed(seed)
    for h in loop.h:
        h.copy_(0.2 * torch.randn(h.shape, generator=g))
    loop.capture()
    calls = args.layers * args.denoise_steps

    def timed(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    for _ in range(args.warmup):
        loop.run_block()
    block_s = timed(loop.run_block, args.steps)
    eager_s = timed(loop.run_block_eager, max(1, args.steps // 4))
    tokens_per_call = cfg["batch"] * cfg["seqlen"]
    per_call = block_s / calls
    flops = shapes.algorithmic_flops(cfg)
    scalar_a = cfg["a_kind"] == 1
    ach = (shapes.ssd_matrix_flops(cfg) if scalar_a else flops) / per_call / 1e12
    peak = PEAK_BF16_MFMA_TFLOPS if scalar_a else PEAK_FP32_VECTOR_TFLOPS
    nbytes = shapes.algorithmic_bytes(cfg) + cfg["batch"] * cfg["d_inner"] * cfg["d_state"] * 4   # + the cached state, read once
    result = {
        "metric": "bidirectional-scan tokens/s/GPU at d_inner=4096,L=8K; HBM GB/s vs peak",
        "value": tokens_per_call / per_call, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": block_s * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "what_a_step_is": "one block: %d denoising steps x %d layers = %d block calls, "
                   "graph replay; value counts the tokens each call scans (batch x G)" % (args.denoise_steps, args.layers, calls),
                   "batch": cfg["batch"], "block_tokens": cfg["seqlen"], "d_inner": cfg["d_inner"], "d_state": cfg["d_state"],
                   "n_heads": cfg["n_heads"], "io_dtype": cfg["io"], "state_dtype": "f32", "layers": args.layers,
                   "denoise_steps": args.denoise_steps},
        "per_call_us": {"graph_replay": per_call * 1e6, "eager": eager_s / calls * 1e6},
        "generated_tokens_per_s": tokens_per_call / block_s,
        "roofline": {"bound": "mfma" if scalar_a else "alu", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                     "frac": ach / peak, "traffic": None,
                     "kernel": "one block call (all its launches), mean over a graph replay of %d calls" % calls,
                     "kernel_ms": per_call * 1e3},
        "hbm": {"achieved": nbytes / per_call / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                "frac": nbytes / per_call / 1e9 / PEAK_HBM_GBPS, "algorithmic_bytes": nbytes},
    }
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle as orc
        npy = lambda d: {k: (None if v is None else v.numpy()) for k, v in d.items()}
        inp = synth.make_inputs(cfg, seed + 100)
        pf, pb = params[0]
        t0 = time.perf_counter()
        reps = 3
        for _ in range(reps):
            orc.bimamba_block_fwd(cfg, npy(pf), npy(pb), npy(inp), h_in=np.zeros((cfg["batch"], cfg["d_inner"], cfg["d_state"])))
        cpu_s = (time.perf_counter() - t0) / reps
        result["cpu_baseline"] = {"value": tokens_per_call / cpu_s, "unit": "tokens/s", "cores": orc.num_threads(),
                                  "kind": "oracle", "seconds": cpu_s, "sample": "one block call of layer 0, whole batch, fp64"}
    print(json.dumps(result))


def bwd_bench(args, torch, bd, shapes, synth):
    """Gradients of the full-sequence path (the paper trains the model, App. A.2): one step is one bimamba_bwd call at
    the headline shape (batch 8, L 8192, d_inner 4096, N 16, bf16 I/O, shared activations, ADD)."""
    cfg = dict(synth.CONFIGS["headline"])
    seed = synth.config_seed(9)
    Bt, L, Dn, N, K, G = (cfg[k] for k in ("batch", "seqlen", "d_inner", "d_state", "d_conv", "n_groups"))
    desc = bd.make_desc(cfg)
    pf, pb = synth.make_params(cfg, seed, 0), synth.make_params(cfg, seed, 1)
    inp = synth.make_inputs(cfg, seed)
    dpf, dpb, dinp = bd.to_device(pf), bd.to_device(pb), bd.to_device(inp, cfg)
    io = bd.io_dtype(cfg)
    g = torch.Generator().manual_seed(seed + 1)
    dout_host = synth.round_io(torch.randn(Bt, L, Dn, generator=g), cfg["io"])
    dout = dout_host.to(device="cuda", dtype=io)
    gi = dict(dx=torch.empty(Bt, L, Dn, dtype=io, device="cuda"), dz=torch.empty(Bt, L, Dn, dtype=io, device="cuda"),
              ddt=torch.empty(Bt, L, Dn, dtype=io, device="cuda"), dB=torch.empty(Bt, L, G, N, device="cuda"),
              dC=torch.empty(Bt, L, G, N, device="cuda"))
    mk = lambda: dict(dconv_w=torch.empty(Dn, K, device="cuda"), dconv_b=torch.empty(Dn, device="cuda"),
                      dA=torch.empty(Dn, N, device="cuda"), dD=torch.empty(Dn, device="cuda"), ddt_bias=torch.empty(Dn, device="cuda"))
    qf, qb = mk(), mk()
    ws = torch.empty(bd.bimamba_bwd_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    call = (desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(dinp), None, bd.make_tensor(dout),
            bd.make_input_grads(gi), None, bd.make_param_grads(qf), bd.make_param_grads(qb), ws)
    for _ in range(args.warmup):
        bd.bimamba_bwd(*call)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        bd.bimamba_bwd(*call)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    flops, nbytes = shapes.algorithmic_flops_bwd(cfg), shapes.algorithmic_bytes_bwd(cfg)
    ach = flops / (ms * 1e-3) / 1e12
    result = {
        "metric": "bidirectional-scan tokens/s/GPU at d_inner=4096,L=8K; HBM GB/s vs peak",
        "value": Bt * L / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "headline_bwd", "what_a_step_is": "one bimamba_bwd call: gradients of the headline forward call",
                   "batch": Bt, "seq_len": L, "d_inner": Dn, "d_state": N, "io_dtype": cfg["io"], "state_dtype": "f32",
                   "inputs": "shared by both directions", "combine": "add",
                   "workspace_bytes": int(ws.numel())},
        "roofline": {"bound": "alu", "achieved": ach, "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                     "frac": ach / PEAK_FP32_VECTOR_TFLOPS, "algorithmic_flops": flops, "traffic": None,
                     "kernel": "bwd_state_kernel + bwd_kernel + bwd_bc_kernel (whole call)", "kernel_ms": ms,
                     "frac_of_unpacked_fp32_peak": ach / PEAK_FP32_UNPACKED_TFLOPS},
        "hbm": {"achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                "frac": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, "algorithmic_bytes": nbytes},
    }
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle as orc
        npy = lambda d: {k: (None if v is None else v.numpy()) for k, v in d.items()}
        sel = list(range(0, Dn, Dn // 64))
        one = dict(cfg, batch=1)
        one_in = {k: v[:1] for k, v in inp.items()}
        t0 = time.perf_counter()
        ref = orc.bimamba_bwd(one, npy(pf), npy(pb), npy(one_in), None, dout_host[:1][..., sel].numpy(), sel=sel)
        cpu_s = time.perf_counter() - t0
        got = gi["dx"][:1][..., sel].float().cpu().numpy().astype(np.float64)
        result["cpu_baseline"] = {"value": L / (cpu_s * Dn / len(sel)), "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                  "seconds": cpu_s, "sample": "batch element 0, all %d tokens, %d of %d channels, fp64 "
                                  "(rate scaled by the channel fraction)" % (L, len(sel), Dn)}
        result["rel_l2_dx_vs_oracle"] = float(np.linalg.norm(got - ref[0]["dx"]) / np.linalg.norm(ref[0]["dx"]))
    print(json.dumps(result))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus %d is not supported: the path shards by batch or "
              "d_inner with no exchange, and no multi-GPU run is part of it)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2511_15927_amd import binding as bd
    from paper_2511_15927_amd import shapes, synth

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read, 1 GiB written per copy
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "3 x copy of 1 GiB", "bytes_read_per_copy": src.numel() * 4,
                          "bytes_written_per_copy": src.numel() * 4}))
        return
    bd.lib()  # fail loudly if the HIP library is not built
    if args.workload.startswith("cfg3_block"):
        return decode_loop_bench(args, torch, bd, shapes, synth)
    if args.workload == "headline_bwd":
        return bwd_bench(args, torch, bd, shapes, synth)
    cfg = dict(synth.CONFIGS[args.workload])
    seed = synth.config_seed(9)
    t0 = time.time()
    pf, pb = synth.make_params(cfg, seed, 0), synth.make_params(cfg, seed, 1)
    if args.general_a:
        pf["A"], pb["A"] = synth.random_A(cfg, seed), synth.random_A(cfg, seed + 1)
    inp = synth.make_inputs(cfg, seed)
    gen_s = time.time() - t0

    desc = bd.make_desc(cfg)
    dpf, dpb, dinp = bd.to_device(pf), bd.to_device(pb), bd.to_device(inp, cfg)
    out = bd.alloc_out(cfg)
    ws = bd.alloc_workspace(desc)
    cpf, cpb, cin, cout = bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(dinp), bd.make_tensor(out)
    stream = torch.cuda.current_stream()

    def step():
        bd.bimamba_fwd(desc, cpf, cpb, cin, None, cout, ws, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # HIP events around the dominant kernel of every timed step (recorded by the library on the launch stream)
    # (every args.probe_every-th step: an event pair on the stream costs the step a few microseconds of its own)
    probed = [i for i in range(args.steps) if i % max(args.probe_every, 1) == 0]
    evs = {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for i in probed}
    for a, b in evs.values():
        a.record(stream)
        b.record(stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i in evs:
            bd.bimamba_profile_next_call(*evs[i])
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    kernel_ms = sum(a.elapsed_time(b) for a, b in evs.values()) / len(evs)

    tokens = cfg["batch"] * cfg["seqlen"]
    value = tokens / (ms_per_step * 1e-3)
    # the same workload with a structure-free A[d, n] (one exponential per state instead of the detected progression)
    general = None
    if not args.general_a and not args.no_general_a and cfg["a_kind"] == 0:
        gpf, gpb = dict(pf), dict(pb)
        gpf["A"], gpb["A"] = synth.random_A(cfg, seed), synth.random_A(cfg, seed + 1)
        dgf, dgb = bd.to_device(gpf), bd.to_device(gpb)
        cgf, cgb = bd.make_params(dgf), bd.make_params(dgb)
        keep = out.clone()
        for _ in range(args.warmup):
            bd.bimamba_fwd(desc, cgf, cgb, cin, None, cout, ws, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            bd.bimamba_fwd(desc, cgf, cgb, cin, None, cout, ws, stream)
        torch.cuda.synchronize()
        gms = (time.perf_counter() - t0) * 1e3 / args.steps
        general = {"value": tokens / (gms * 1e-3), "unit": "tokens/s", "ms_per_step": gms}
        out.copy_(keep)
    flops = shapes.algorithmic_flops(cfg)
    nbytes = shapes.algorithmic_bytes(cfg)
    ach_tflops = flops / (kernel_ms * 1e-3) / 1e12
    ach_gbps = nbytes / (kernel_ms * 1e-3) / 1e9
    scalar_a = cfg["a_kind"] == 1
    ssd = scalar_a and cfg["io"] == "bf16" and cfg["d_state"] in (64, 128) and cfg["d_inner"] // cfg["n_heads"] in (32, 64)
    kernel = "sweep_kernel<N=%d,%s,%s>" % (cfg["d_state"], "scalarA" if scalar_a else "perStateA", cfg["io"])
    roofline = {"bound": "alu", "achieved": ach_tflops, "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                "frac": ach_tflops / PEAK_FP32_VECTOR_TFLOPS, "algorithmic_flops": flops}
    if ssd:
        # the chunked matrix-core kernels: one launch per direction, both inside the probed interval
        # one time part and several chunks: the sixteen-wave form; otherwise the eight-wave form (+ state and carry kernels)
        form = "ssd_wide_kernel" if bd.bimamba_time_chunks(desc) == 1 and cfg["seqlen"] > 64 else "ssd_kernel"
        kernel = "%s<N=%d,P=%d> (two launches, one per direction)" % (form, cfg["d_state"], cfg["d_inner"] // cfg["n_heads"])
        mflops = shapes.ssd_matrix_flops(cfg)
        ach = mflops / (kernel_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / PEAK_BF16_MFMA_TFLOPS, "algorithmic_flops": mflops}
    counters, profile_kernel, profile_file = read_profile("sweep_" + args.workload)
    # the chunked path runs one launch per direction, both inside the probed interval; the summary holds one launch's mean
    traffic = traffic_of(counters, 2 if ssd else 1)
    simds = 4 * torch.cuda.get_device_properties(0).multi_processor_count
    valu_busy, waves_per_simd = valu_busy_of(counters, simds)
    clock_ghz, valu_busy_own_clock = sustained_clock_of(counters, simds)
    ceiling = copy_ceiling_gbps(torch)
    roofline.update({"traffic": traffic, "kernel": kernel, "kernel_ms": kernel_ms,
                     "traffic_source": {"stored_profile": profile_file, "profiled_kernel": profile_kernel,
                                        "note": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command, "
                                                "scaled by the 1 GiB copy calibration in the same file"},
                     "valu_busy_from_profile": valu_busy, "resident_waves_per_simd_from_profile": waves_per_simd,
                     "sustained_clock_ghz_from_profile": clock_ghz, "valu_busy_at_sustained_clock": valu_busy_own_clock,
                     # 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz: what fp32 code without packed instructions can issue
                     "frac_of_unpacked_fp32_peak": None if roofline["bound"] != "alu" else
                     roofline["achieved"] / PEAK_FP32_UNPACKED_TFLOPS})
    result = {
        "metric": "bidirectional-scan tokens/s/GPU at d_inner=4096,L=8K; HBM GB/s vs peak",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "batch": cfg["batch"], "seq_len": cfg["seqlen"], "d_inner": cfg["d_inner"],
                   "d_state": cfg["d_state"], "n_heads": cfg["n_heads"], "io_dtype": cfg["io"], "state_dtype": "f32",
                   "A": "general" if args.general_a else ("scalar per head" if scalar_a else
                                                           "-(1..N) per state (arithmetic in n: detected on the device)"),
                   "inputs": "shared by both directions",
                   "combine": "add", "time_chunks": bd.bimamba_time_chunks(desc)},
        "roofline": roofline,
        "hbm": {"achieved": ach_gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": ach_gbps / PEAK_HBM_GBPS,
                "algorithmic_bytes": nbytes, "copy_ceiling_measured": ceiling, "frac_of_copy_ceiling": ach_gbps / ceiling},
        "general_A": general,
        "input_generation_s": gen_s,
    }

    if not args.no_cpu_baseline:
        import numpy as np
        import oracle as orc
        nb = max(1, min(args.cpu_batches, cfg["batch"]))
        sub = dict(cfg, batch=nb)
        npy = lambda d: {k: (None if v is None else v.numpy()) for k, v in d.items()}
        sub_in = {k: v[:nb].contiguous() for k, v in inp.items()}
        t0 = time.perf_counter()
        ref = orc.bimamba_fwd(sub, npy(pf), npy(pb), npy(sub_in))
        cpu_s = time.perf_counter() - t0
        got = out[:nb].float().cpu().numpy().astype(np.float64)
        err = max(float(np.linalg.norm(got[b] - ref[b]) / np.linalg.norm(ref[b])) for b in range(nb))
        # the same oracle on one thread, on a sample sized to a few seconds: the first 256 channels of batch element 0
        threads = orc.num_threads()
        one_sel = list(range(min(256, cfg["d_inner"])))
        one_in = {k: v[:1].contiguous() for k, v in inp.items()}
        orc.set_num_threads(1)
        t0 = time.perf_counter()
        orc.bimamba_fwd(dict(cfg, batch=1), npy(pf), npy(pb), npy(one_in), sel=one_sel)
        one_s = time.perf_counter() - t0
        orc.set_num_threads(threads)
        one_rate = cfg["seqlen"] * (len(one_sel) / cfg["d_inner"]) / one_s
        result["cpu_baseline"] = {"value": nb * cfg["seqlen"] / cpu_s, "unit": "tokens/s", "cores": threads,
                                  "kind": "oracle", "seconds": cpu_s,
                                  "sample": "batch elements 0..%d of %d, all %d tokens and %d channels, fp64" % (
                                      nb - 1, cfg["batch"], cfg["seqlen"], cfg["d_inner"]),
                                  "single_thread": {"value": one_rate, "unit": "tokens/s", "cores": 1, "seconds": one_s,
                                                    "sample": "batch element 0, all %d tokens, %d of %d channels "
                                                              "(rate scaled by the channel fraction)" % (
                                                                  cfg["seqlen"], len(one_sel), cfg["d_inner"])}}
        result["rel_l2_vs_oracle"] = err
    print(json.dumps(result))


if __name__ == "__main__":
    main()
