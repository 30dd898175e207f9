"""Block-diffusion decode loop around bimamba_block_fwd (paper Sec. 4.3, block-cache decoding).

A block of G tokens is denoised in n_steps = G / p steps (Sec. 4.3 throughput set-up: p tokens per step); at every
step all n_layers mixer layers re-scan the block from their cached forward state, the reverse scan staying inside the
block; the last step commits each layer's state and conv tail, which the next block starts from.  This module only
sequences library calls and owns the buffers: every scan runs in the HIP library.

Layer chaining of this benchmark stack (no projections between the mixers are part of the path): layer l's output is
layer l+1's x; z, dt, B, C of a step are shared by the layers; parameters are per layer and per direction.

The n_steps x n_layers calls of a block are captured ONCE into a HIP graph (torch.cuda.CUDAGraph: stream capture of
the library's launches, which contain no memset nodes) and replayed per block; the caller refreshes the static step
inputs between replays.  Why there is no kernel that keeps h on chip across the steps of a block: step s + 1 of a layer
consumes what the whole network made of step s (in the paper's model through the projections and MLPs, here through
the 23 other layers), so between two steps of one layer every other layer has to run; the state of all layers
(n_layers x batch x d_inner x d_state fp32, 100 MB at batch 16) exceeds what registers and LDS hold, so it lives in
HBM/L2 between calls and a call reads it once (4 MB per layer call against 8 MB of activations).
"""
import torch

from . import binding as bd
from . import synth


class BlockDecodeLoop:
    def __init__(self, cfg, layer_params, n_steps, keep_layer_outputs=False, static_scratch=False, device="cuda"):
        """cfg: block config (seqlen = G); layer_params: list of (params_f, params_b) dicts of CPU float32 tensors."""
        self.cfg, self.n_layers, self.n_steps = dict(cfg), len(layer_params), int(n_steps)
        self.desc = bd.make_desc(cfg)
        Bt, G, Dn, N, K = cfg["batch"], cfg["seqlen"], cfg["d_inner"], cfg["d_state"], cfg["d_conv"]
        io = bd.io_dtype(cfg)
        tail_ch = synth.conv_channels(cfg)
        self._dev_params = [(bd.to_device(pf, device=device), bd.to_device(pb, device=device)) for pf, pb in layer_params]
        self._params = [(bd.make_params(f), bd.make_params(b)) for f, b in self._dev_params]
        self.h = [torch.zeros(Bt, Dn, N, dtype=torch.float32, device=device) for _ in range(self.n_layers)]
        self.tail = [torch.zeros(Bt, max(K - 1, 1), tail_ch, dtype=io, device=device)[:, :K - 1].contiguous()
                     for _ in range(self.n_layers)]
        H, GN = cfg["n_heads"], cfg["n_groups"] * N
        # static inputs of each step (the caller writes the block's current tokens here before a block runs)
        self.step_inputs = [dict(x=torch.zeros(Bt, G, Dn, dtype=io, device=device), z=torch.zeros(Bt, G, Dn, dtype=io, device=device),
                                 dt=torch.zeros(Bt, G, H, dtype=io, device=device), B=torch.zeros(Bt, G, GN, dtype=io, device=device),
                                 C=torch.zeros(Bt, G, GN, dtype=io, device=device)) for _ in range(self.n_steps)]
        width = Dn * (2 if cfg["combine"] == bd.COMBINE_SEPARATE else 1)
        assert width == Dn, "layers chain out -> x, which needs the additive combine"
        n_act = self.n_steps * self.n_layers if keep_layer_outputs else 2
        self._act = [torch.zeros(Bt, G, Dn, dtype=io, device=device) for _ in range(n_act)]
        self.keep = keep_layer_outputs
        self.out = [torch.zeros(Bt, G, Dn, dtype=io, device=device) for _ in range(self.n_steps)]   # last layer, per step
        self.static_scratch = static_scratch
        self.ws = None if static_scratch else bd.alloc_workspace(self.desc, 1, device=device)
        self._graph = None

    def layer_output(self, step, layer):
        assert self.keep
        return self.out[step] if layer == self.n_layers - 1 else self._act[step * self.n_layers + layer]

    def set_step_inputs(self, step, inputs):
        """inputs: dict of tensors x, z [Bt,G,Dn]; dt [Bt,G,H]; B, C [Bt,G,G*N] or [Bt,G,groups,N] (any device)."""
        for k, dst in self.step_inputs[step].items():
            dst.copy_(inputs[k].reshape(dst.shape))

    def _call(self, layer, step, x, out, commit, stream):
        pf, pb = self._params[layer]
        si = self.step_inputs[step]
        ins = bd.make_inputs(dict(x=x, z=si["z"], dt=si["dt"], B=si["B"], C=si["C"]))
        h, tail = self.h[layer], self.tail[layer]
        has_tail = tail.shape[1] > 0
        a = (self.desc, pf, pb, ins, None, h, tail if has_tail else None, h if commit else None,
             tail if (commit and has_tail) else None, bd.make_tensor(out))
        if self.static_scratch:
            bd.bimamba_block_fwd_static(*a, stream=stream)
        else:
            bd.bimamba_block_fwd(*a, self.ws, stream=stream)

    def run_block_eager(self, stream=None):
        """All steps of one block, launch by launch; the last step commits every layer's state and conv tail in place."""
        for step in range(self.n_steps):
            commit = step == self.n_steps - 1
            x = self.step_inputs[step]["x"]
            for layer in range(self.n_layers):
                last = layer == self.n_layers - 1
                out = self.out[step] if last else (self._act[step * self.n_layers + layer] if self.keep else self._act[layer & 1])
                self._call(layer, step, x, out, commit, stream)
                x = out

    def capture(self):
        """Capture one block's calls into a graph (after one eager pass on a side stream, so that no kernel variant
        is launched for the first time under capture and the cache is left as it was)."""
        saved = [(h.clone(), t.clone()) for h, t in zip(self.h, self.tail)]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.run_block_eager()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for (h0, t0), h, t in zip(saved, self.h, self.tail):
            h.copy_(h0)
            t.copy_(t0)
        self._graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self._graph):
            self.run_block_eager()
        # the capture itself does not run the kernels: the cache is untouched
        return self

    def run_block(self):
        """Replay the captured block (capture() first)."""
        self._graph.replay()

    def prefill(self, make_layer_inputs, prefix_len):
        """Scan a clean prefix once through every layer, committing each layer's state and conv tail.
        make_layer_inputs: dict of device tensors for the prefix (x of layer 0, z, dt, B, C)."""
        cfg_p = dict(self.cfg, seqlen=prefix_len)
        desc = bd.make_desc(cfg_p)
        ws = bd.alloc_workspace(desc, 1)
        x = make_layer_inputs["x"]
        for layer in range(self.n_layers):
            pf, pb = self._params[layer]
            out = torch.empty_like(make_layer_inputs["x"])
            ins = bd.make_inputs(dict(make_layer_inputs, x=x))
            tail = self.tail[layer]
            bd.bimamba_block_fwd(desc, pf, pb, ins, None, None, None, self.h[layer], tail if tail.shape[1] > 0 else None,
                                 bd.make_tensor(out), ws)
            x = out
        torch.cuda.synchronize()
        return x
