"""Seeded synthetic inputs and parameters for the bidirectional Mamba mixer path.

This module serves both the HIP path and the CPU oracle and contains none of the
mixer's arithmetic: it only draws tensors of the shapes and value distributions of
the paper's workloads (App. A model/hyper-parameter tables: d_inner = 2 d_model,
conv width 4, lengths 64..65K, batch 1 or 8, block length 32) and rounds them once
to the I/O dtype, so that both sides receive bit-identical values.

Everything is CPU torch with an explicit generator; draw order is fixed:
x, z, dt_noise, dt_shift, B, C for inputs; conv_w, conv_b, D, A, dt_bias for each
direction's parameters.
"""
import math

import torch

A_PER_HEAD_STATE, A_SCALAR_PER_HEAD = 0, 1
D_PER_CHANNEL, D_PER_HEAD = 0, 1
COMBINE_ADD, COMBINE_SEPARATE = 0, 1
BASE_SEED = 20251115


def mixer_cfg(batch, seqlen, d_inner, d_state=16, n_heads=None, n_groups=1, d_conv=4, io="bf16",
              a_kind=A_PER_HEAD_STATE, d_kind=D_PER_CHANNEL, dt_softplus=0, conv_bc=0, combine=COMBINE_ADD,
              time_chunks=0, state_split=0):
    """Shape/mode descriptor as a plain dict (keys mirror the C descriptor)."""
    return dict(batch=batch, seqlen=seqlen, d_inner=d_inner, d_state=d_state,
                n_heads=d_inner if n_heads is None else n_heads, n_groups=n_groups, d_conv=d_conv, io=io,
                a_kind=a_kind, d_kind=d_kind, dt_softplus=dt_softplus, conv_bc=conv_bc, combine=combine,
                time_chunks=time_chunks, state_split=state_split)


def m2_cfg(batch, seqlen, d_inner, headdim=64, d_state=128, io="bf16", **kw):
    """The paper's Mamba-2 parameterisation: scalar A and D per head, dt per head, one B/C group,
    B and C pass through the short conv together with x, dt = softplus(raw + bias)."""
    base = dict(n_heads=d_inner // headdim, n_groups=1, a_kind=A_SCALAR_PER_HEAD, d_kind=D_PER_HEAD,
                dt_softplus=1, conv_bc=1)
    base.update(kw)
    return mixer_cfg(batch, seqlen, d_inner, d_state=d_state, io=io, **base)


# The benchmark configurations (selective-scan shapes first, Mamba-2 shapes beside them).
CONFIGS = {
    "cfg0": mixer_cfg(1, 256, 512, io="f32"),
    "cfg0_m2": m2_cfg(1, 256, 512, headdim=64, d_state=128, io="f32"),
    "cfg1": mixer_cfg(8, 2048, 4096),
    "cfg1_m2": m2_cfg(8, 2048, 4096),
    "cfg2": mixer_cfg(1, 32768, 4096),
    "cfg2_m2": m2_cfg(1, 32768, 4096),
    "cfg3_prefix": mixer_cfg(16, 4096, 4096),
    "cfg3_block": mixer_cfg(16, 32, 4096),
    "cfg3_block_m2": m2_cfg(16, 32, 4096),
    "headline": mixer_cfg(8, 8192, 4096),
    "headline_b1": mixer_cfg(1, 8192, 4096),
    "headline_m2": m2_cfg(8, 8192, 4096),
    "paper_1p3b": m2_cfg(1, 1024, 3840, headdim=32, d_state=128),
}
CFG4_BATCHES = (1, 8, 32, 64)
CFG4_LENGTHS = (1024, 4096, 8192)
CFG4_LAYERS = 24


def cfg4(batch, seqlen):
    return mixer_cfg(batch, seqlen, 2048)


def conv_channels(cfg):
    return cfg["d_inner"] + (2 * cfg["n_groups"] * cfg["d_state"] if cfg["conv_bc"] else 0)


def round_io(t, io):
    """Round once to the I/O dtype and return float32 holding exactly those values."""
    if io == "bf16":
        return t.to(torch.bfloat16).to(torch.float32)
    return t.to(torch.float32)


def _gen(seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def make_inputs(cfg, seed, seqlen=None):
    """x, z [Bt,L,Dn]; dt [Bt,L,H]; B, C [Bt,L,G,N]; float32 tensors holding I/O-dtype values.

    dt is Delta itself (softplus already applied) unless cfg['dt_softplus'], in which case it is the raw
    pre-activation and the per-head shift is returned by make_params as dt_bias of each direction
    (both directions share the shift drawn here so that Delta has the recipe's distribution).
    """
    g = _gen(seed)
    Bt, L = cfg["batch"], cfg["seqlen"] if seqlen is None else seqlen
    Dn, N, H, G = cfg["d_inner"], cfg["d_state"], cfg["n_heads"], cfg["n_groups"]
    io = cfg["io"]
    x = torch.randn(Bt, L, Dn, generator=g)
    z = torch.randn(Bt, L, Dn, generator=g)
    noise = 0.5 * torch.randn(Bt, L, H, generator=g)
    shift = dt_shift(cfg, seed)
    if cfg["dt_softplus"]:
        dt = noise
    else:
        dt = torch.nn.functional.softplus((noise + shift).double()).float()
    Bm = torch.randn(Bt, L, G, N, generator=g)
    Cm = torch.randn(Bt, L, G, N, generator=g)
    return dict(x=round_io(x, io), z=round_io(z, io), dt=round_io(dt, io), B=round_io(Bm, io), C=round_io(Cm, io))


def dt_shift(cfg, seed):
    """Per-Delta-channel shift b with softplus(b) log-uniform in [1e-3, 1e-1]."""
    g = _gen(int(seed) * 7919 + 17)
    H = cfg["n_heads"]
    target = torch.exp(torch.empty(H, dtype=torch.float64).uniform_(math.log(1e-3), math.log(1e-1), generator=g))
    return torch.log(torch.expm1(target)).float()   # inverse softplus


def make_params(cfg, seed, direction):
    """Per-direction parameters (untied): conv_w [C,K], conv_b [C], D, A, dt_bias; float32."""
    g = _gen(int(seed) * 2 + 1000003 * (1 + int(direction)))
    Dn, N, H, K = cfg["d_inner"], cfg["d_state"], cfg["n_heads"], cfg["d_conv"]
    Cc = conv_channels(cfg)
    conv_w = 0.5 * torch.randn(Cc, K, generator=g)
    conv_b = 0.1 * torch.randn(Cc, generator=g)
    D = torch.rand(H if cfg["d_kind"] == D_PER_HEAD else Dn, generator=g)
    if cfg["a_kind"] == A_PER_HEAD_STATE:
        A = -torch.arange(1, N + 1, dtype=torch.float32).repeat(H, 1)     # A = -exp(A_log), A_log = log(1..N)
    else:
        A = -(1.0 + 15.0 * torch.rand(H, generator=g))
    p = dict(conv_w=conv_w.contiguous(), conv_b=conv_b.contiguous(), D=D.contiguous(), A=A.contiguous(), dt_bias=None)
    if cfg["dt_softplus"]:
        p["dt_bias"] = dt_shift(cfg, seed).contiguous()
    return p


def random_A(cfg, seed):
    """General per-(head,state) A with no structure across states: -exp(U(ln 0.5, ln 16))."""
    g = _gen(int(seed) * 31 + 5)
    H, N = cfg["n_heads"], cfg["d_state"]
    if cfg["a_kind"] == A_PER_HEAD_STATE:
        return -torch.exp(torch.empty(H, N).uniform_(math.log(0.5), math.log(16.0), generator=g))
    return -torch.exp(torch.empty(H).uniform_(math.log(0.5), math.log(16.0), generator=g))


def config_seed(index, layer=0):
    return BASE_SEED + 1000 * int(index) + int(layer)
