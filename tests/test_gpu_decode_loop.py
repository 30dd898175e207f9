"""The block-diffusion decode loop (Sec. 4.3): n_layers x n_steps block calls per block, captured once as a HIP graph
and replayed per block.  Every layer call of every step is checked against the fp64 oracle fed that call's own input
(layer by layer), the committed caches against the oracle's chain, and graph replays against eager runs bit for bit
(several replays, with eager work and synchronisation between them)."""
import numpy as np
import pytest
import torch

from helpers import assert_close, rel_l2, to_np
from paper_2511_15927_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("layout,G,static", [("selective", 32, False), ("selective", 64, True), ("mamba2", 32, False),
                                             ("mamba2", 128, False)])
def test_decode_loop_graph_matches_oracle_layer_by_layer(oracle, layout, G, static):
    from paper_2511_15927_amd import binding as bd
    from paper_2511_15927_amd.decode import BlockDecodeLoop
    assert torch.cuda.is_available(), "these tests need the MI355X"
    n_layers, n_steps, n_blocks = 3, 2, 3
    if layout == "selective":
        cfg, h_tol = synth.mixer_cfg(2, G, 192), 1e-5
    else:
        cfg, h_tol = synth.m2_cfg(2, G, 128, headdim=32, d_state=64), 1e-2
    Bt, Dn, N, K = cfg["batch"], cfg["d_inner"], cfg["d_state"], cfg["d_conv"]
    params = [(synth.make_params(cfg, 3000 + l, 0), synth.make_params(cfg, 3000 + l, 1)) for l in range(n_layers)]
    loop = BlockDecodeLoop(cfg, params, n_steps, keep_layer_outputs=True, static_scratch=static)
    g = torch.Generator().manual_seed(G)
    h_ref, tail_ref = [], []
    for l in range(n_layers):        # a cache as some earlier blocks might have left it
        h0 = (0.2 * torch.randn(Bt, Dn, N, generator=g)).float()
        t0 = synth.round_io(torch.randn(Bt, K - 1, synth.conv_channels(cfg), generator=g), cfg["io"])
        loop.h[l].copy_(h0)
        loop.tail[l].copy_(t0)
        h_ref.append(h0.numpy().astype(np.float64))
        tail_ref.append(t0.numpy().astype(np.float64))
    loop.capture()
    for blk in range(n_blocks):
        steps = [synth.make_inputs(cfg, 3100 + 10 * blk + s) for s in range(n_steps)]
        for s in range(n_steps):
            loop.set_step_inputs(s, steps[s])
        saved = [(h.clone(), t.clone()) for h, t in zip(loop.h, loop.tail)]
        torch.cuda.synchronize()
        loop.run_block()
        torch.cuda.synchronize()
        got = [[loop.layer_output(s, l).float().cpu().numpy() for l in range(n_layers)] for s in range(n_steps)]
        cache = [(h.clone(), t.clone()) for h, t in zip(loop.h, loop.tail)]
        # the same block, launch by launch, from the same cache: bit-identical outputs and caches
        for (h0, t0), h, t in zip(saved, loop.h, loop.tail):
            h.copy_(h0)
            t.copy_(t0)
        loop.run_block_eager()
        torch.cuda.synchronize()
        for s in range(n_steps):
            for l in range(n_layers):
                assert np.array_equal(got[s][l], loop.layer_output(s, l).float().cpu().numpy()), (blk, s, l)
        for (h1, t1), h, t in zip(cache, loop.h, loop.tail):
            assert torch.equal(h1, h) and torch.equal(t1, t), blk
        # the oracle, layer by layer, fed each call's own input
        for s in range(n_steps):
            for l in range(n_layers):
                x_in = steps[s]["x"].numpy() if l == 0 else got[s][l - 1]
                ins = dict(to_np(steps[s]), x=x_in)
                ref, h_new, t_new = oracle.bimamba_block_fwd(cfg, to_np(params[l][0]), to_np(params[l][1]), ins,
                                                             h_in=h_ref[l], tail_in=tail_ref[l])
                assert_close(got[s][l], ref, 2e-2, (blk, s, l))
                if s == n_steps - 1:
                    h_ref[l], tail_ref[l] = h_new, t_new
        for l in range(n_layers):
            assert rel_l2(loop.h[l].cpu().numpy(), h_ref[l]) < h_tol, (blk, l)
            assert np.array_equal(loop.tail[l].float().cpu().numpy().astype(np.float64), tail_ref[l]), (blk, l)


def test_decode_loop_prefill_then_blocks_equals_full_forward_scan(oracle):
    """One layer: a prefix scanned once, then committed blocks; the final cached state equals the oracle's forward
    scan of prefix || committed blocks (the block-cache statement of Sec. 4.3 through the loop component)."""
    from paper_2511_15927_amd import binding as bd
    from paper_2511_15927_amd.decode import BlockDecodeLoop
    cfg = synth.mixer_cfg(2, 32, 96)
    pf, pb = synth.make_params(cfg, 3300, 0), synth.make_params(cfg, 3300, 1)
    loop = BlockDecodeLoop(cfg, [(pf, pb)], n_steps=4)
    prefix = synth.make_inputs(cfg, 3301, seqlen=77)
    loop.prefill(bd.to_device({k: v.reshape(v.shape[0], v.shape[1], -1) for k, v in prefix.items()}, cfg), 77)
    loop.capture()
    committed = [to_np(prefix)]
    for blk in range(3):
        for s in range(4):
            inp = synth.make_inputs(cfg, 3310 + 10 * blk + s)
            loop.set_step_inputs(s, inp)
        committed.append(to_np(inp))              # the last step's tokens are the ones committed
        loop.run_block()
    torch.cuda.synchronize()
    whole = {k: np.concatenate([c[k] for c in committed], axis=1) for k in ("x", "z", "dt", "B", "C")}
    _, h_full = oracle.one_direction(dict(cfg, seqlen=77 + 3 * 32), to_np(pf), whole, +1)
    assert rel_l2(loop.h[0].cpu().numpy(), h_full) < 1e-5
    assert np.array_equal(loop.tail[0].float().cpu().numpy(), whole["x"][:, -3:])
