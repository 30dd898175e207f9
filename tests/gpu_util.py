"""GPU-side test helpers: run the HIP path through the C ABI and bring results back as numpy float64."""
import numpy as np
import torch

from paper_2511_15927_amd import binding as bd

TOL = {"f32": 1e-5, "bf16": 2e-2}     # max relative L2 error against the fp64 oracle, per batch element


def to_t(d):
    return {k: (None if v is None else torch.as_tensor(v)) for k, v in d.items()}


def gpu_fwd(cfg, pf, pb, in_f, in_b=None, **desc_override):
    """bimamba_fwd on cuda:0.  pf/pb/in_*: dicts of CPU float32 tensors (or numpy).  Returns float64 numpy out."""
    desc = bd.make_desc(cfg, **desc_override)
    c = dict(cfg, **desc_override)
    dpf, dpb = bd.to_device(to_t(pf)), bd.to_device(to_t(pb))
    dif = bd.to_device(to_t(in_f), c)
    dib = None if in_b is None else bd.to_device(to_t(in_b), c)
    out = bd.alloc_out(c)
    ws = bd.alloc_workspace(desc)
    bd.bimamba_fwd(desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(dif),
                   None if dib is None else bd.make_inputs(dib), bd.make_tensor(out), ws)
    torch.cuda.synchronize()
    res = out.float().cpu().numpy().astype(np.float64)
    if c["combine"] == bd.COMBINE_SEPARATE:
        res = res.reshape(c["batch"], c["seqlen"], 2, c["d_inner"])
    return res


def gpu_block_fwd(cfg, pf, pb, in_f, in_b=None, h_in=None, tail_in=None, commit=True, **desc_override):
    """bimamba_block_fwd on cuda:0.  h_in: float32 tensor/array [Bt,Dn,N]; tail_in: [Bt,K-1,tail_ch] values
    representable in the I/O dtype.  Returns (out, h_out, tail_out) as float64 numpy (None when not committed)."""
    desc = bd.make_desc(cfg, **desc_override)
    c = dict(cfg, **desc_override)
    dpf, dpb = bd.to_device(to_t(pf)), bd.to_device(to_t(pb))
    dif = bd.to_device(to_t(in_f), c)
    dib = None if in_b is None else bd.to_device(to_t(in_b), c)
    out = bd.alloc_out(c)
    ws = bd.alloc_workspace(desc, 1)
    Bt, Dn, N, K = c["batch"], c["d_inner"], c["d_state"], c["d_conv"]
    tail_ch = Dn + (2 * c["n_groups"] * N if c["conv_bc"] else 0)
    dh_in = None if h_in is None else torch.as_tensor(h_in, dtype=torch.float32).cuda().contiguous()
    dt_in = None if tail_in is None else torch.as_tensor(tail_in).to(device="cuda", dtype=bd.io_dtype(c)).contiguous()
    dh_out = torch.full((Bt, Dn, N), float("nan"), dtype=torch.float32, device="cuda") if commit else None
    dt_out = torch.full((Bt, max(K - 1, 1), tail_ch), float("nan"), dtype=bd.io_dtype(c), device="cuda")[:, :K - 1] \
        .contiguous() if commit else None
    bd.bimamba_block_fwd(desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(dif),
                         None if dib is None else bd.make_inputs(dib), dh_in, dt_in, dh_out, dt_out,
                         bd.make_tensor(out), ws)
    torch.cuda.synchronize()
    res = out.float().cpu().numpy().astype(np.float64)
    if c["combine"] == bd.COMBINE_SEPARATE:
        res = res.reshape(Bt, c["seqlen"], 2, Dn)
    h = None if dh_out is None else dh_out.cpu().numpy().astype(np.float64)
    t = None if dt_out is None else dt_out.float().cpu().numpy().astype(np.float64)
    return res, h, t


def gpu_bwd(cfg, pf, pb, in_f, in_b, dout):
    """bimamba_bwd on cuda:0.  dout: array shaped like gpu_fwd's result (values representable in the I/O dtype).
    Returns (din_f, din_b, dparams_f, dparams_b) as dicts of float64 numpy arrays, named as in oracle.bimamba_bwd."""
    desc = bd.make_desc(cfg)
    Bt, L, Dn, N, H, G, K = (cfg[k] for k in ("batch", "seqlen", "d_inner", "d_state", "n_heads", "n_groups", "d_conv"))
    io = bd.io_dtype(cfg)
    dpf, dpb = bd.to_device(to_t(pf)), bd.to_device(to_t(pb))
    dif = bd.to_device(to_t(in_f), cfg)
    dib = None if in_b is None else bd.to_device(to_t(in_b), cfg)
    do = torch.as_tensor(np.asarray(dout)).reshape(Bt, L, Dn * (2 if cfg["combine"] == bd.COMBINE_SEPARATE else 1)) \
        .to(device="cuda", dtype=io).contiguous()

    def input_grads():
        nan = float("nan")
        return dict(dx=torch.full((Bt, L, Dn), nan, dtype=io, device="cuda"), dz=torch.full((Bt, L, Dn), nan, dtype=io, device="cuda"),
                    ddt=torch.full((Bt, L, H), nan, dtype=io, device="cuda"),
                    dB=torch.full((Bt, L, G, N), nan, dtype=torch.float32, device="cuda"),
                    dC=torch.full((Bt, L, G, N), nan, dtype=torch.float32, device="cuda"))

    def param_grads():
        nan = float("nan")
        f = lambda *s: torch.full(s, nan, dtype=torch.float32, device="cuda")
        return dict(dconv_w=f(Dn, K), dconv_b=f(Dn), dA=f(H, N), dD=f(Dn), ddt_bias=f(H))

    gf, gb = input_grads(), (None if in_b is None else input_grads())
    qf, qb = param_grads(), param_grads()
    ws = torch.empty(max(bd.bimamba_bwd_workspace_bytes(desc), 16), dtype=torch.uint8, device="cuda")
    bd.bimamba_bwd(desc, bd.make_params(dpf), bd.make_params(dpb), bd.make_inputs(dif),
                   None if dib is None else bd.make_inputs(dib), bd.make_tensor(do), bd.make_input_grads(gf),
                   None if gb is None else bd.make_input_grads(gb), bd.make_param_grads(qf), bd.make_param_grads(qb), ws)
    torch.cuda.synchronize()
    host = lambda d: None if d is None else {k: v.float().cpu().numpy().astype(np.float64) for k, v in d.items()}
    return host(gf), host(gb), host(qf), host(qb)
