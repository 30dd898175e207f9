"""Child process of test_first_call_in_a_process_captured_into_a_graph: the very first library call of this process is
made under stream capture, so every first-use set-up the library does for a kernel (occupancy and attribute queries,
raising the dynamic-LDS limit) happens inside the capture.  Replays are checked against the fp64 oracle and against an
eager call made afterwards; prints one JSON line."""
import json
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))


def main(layout):
    import oracle as orc
    from helpers import rel_l2, to_np
    from paper_2511_15927_amd import binding as bd
    from paper_2511_15927_amd import synth
    cfg = synth.mixer_cfg(3, 32, 200, d_state=8) if layout == "selective" else synth.m2_cfg(3, 40, 128, headdim=32, d_state=64)
    N, K, Bt, Dn = cfg["d_state"], cfg["d_conv"], cfg["batch"], cfg["d_inner"]
    pf, pb, inp = synth.make_params(cfg, 5, 0), synth.make_params(cfg, 5, 1), synth.make_inputs(cfg, 5)
    g = torch.Generator().manual_seed(9)
    h0 = (0.2 * torch.randn(Bt, Dn, N, generator=g)).float()
    tail0 = synth.round_io(torch.randn(Bt, K - 1, synth.conv_channels(cfg), generator=g), "bf16")
    dpf, dpb, dinp = bd.to_device(pf), bd.to_device(pb), bd.to_device(inp, cfg)
    cpf, cpb, cin = bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(dinp)
    desc = bd.make_desc(cfg)
    h_in, tail_in = h0.cuda(), tail0.to(torch.bfloat16).cuda()
    h_out, tail_out = torch.zeros_like(h_in), torch.zeros_like(tail_in)
    out, ws = bd.alloc_out(cfg), bd.alloc_workspace(desc, 1)
    out.zero_()
    c_out = bd.make_tensor(out)

    def call():
        bd.bimamba_block_fwd(desc, cpf, cpb, cin, None, h_in, tail_in, h_out, tail_out, c_out, ws)

    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):          # no library call has been made in this process before this one
        call()
    ref, h_ref, t_ref = orc.bimamba_block_fwd(cfg, to_np(pf), to_np(pb), to_np(inp), h_in=h0.numpy(), tail_in=tail0.numpy())
    res = {"layout": layout, "replays": []}
    for rep in range(3):
        out.zero_(); h_out.zero_(); tail_out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        res["replays"].append({"out": rel_l2(out.float().cpu().numpy(), ref), "h": rel_l2(h_out.cpu().numpy(), h_ref),
                               "tail_equal": bool(np.array_equal(tail_out.float().cpu().numpy().astype(np.float64), t_ref))})
        kept = (out.clone(), h_out.clone(), tail_out.clone())
    out.zero_(); h_out.zero_(); tail_out.zero_()
    call()
    torch.cuda.synchronize()
    res["eager_equals_replay"] = bool(torch.equal(out, kept[0]) and torch.equal(h_out, kept[1]) and torch.equal(tail_out, kept[2]))
    print(json.dumps(res))


if __name__ == "__main__":
    main(sys.argv[1])
