"""Shape bookkeeping for the mixer path: channel counts, the paper's per-token FLOP convention (App. C, Mamba-2
layer table) and the algorithmic byte / flop counts used by the benchmark's roofline."""


def conv_channels(d_inner, n_groups, d_state, conv_bc):
    return d_inner + (2 * n_groups * d_state if conv_bc else 0)


def in_proj_width(d_inner, n_groups, d_state, n_heads):
    """Width of the projection that produces z, x, B, C, dt for one direction (the paper's D_in)."""
    return 2 * d_inner + 2 * n_groups * d_state + n_heads


def paper_flops_per_token(d_model, d_inner, d_state, d_conv, n_heads, n_groups=1):
    """Per-token forward FLOPs of one direction of the paper's Mamba-2 layer, by its counting conventions
    (2mn per linear layer, scan 2*d_inner*d_state, conv conv_ch*d_conv)."""
    d_in = in_proj_width(d_inner, n_groups, d_state, n_heads)
    conv_ch = conv_channels(d_inner, n_groups, d_state, 1)
    parts = dict(in_proj=2 * d_model * d_in, conv=conv_ch * d_conv, scan=2 * d_inner * d_state,
                 out_proj=2 * d_inner * d_model)
    parts["one_direction"] = sum(parts.values())
    parts["bidirectional"] = 2 * parts["one_direction"]
    return parts


def algorithmic_bytes(cfg, shared_inputs=True):
    """Bytes the path must move once per call: each input read once, the output written once (state, tail and
    parameters excluded).  Token-channel activations dominate; B and C amortise over d_inner."""
    e = 2 if cfg["io"] == "bf16" else 4
    Bt, L, Dn, H, GN = cfg["batch"], cfg["seqlen"], cfg["d_inner"], cfg["n_heads"], cfg["n_groups"] * cfg["d_state"]
    ndir = 1 if shared_inputs else 2
    reads = ndir * (2 * Dn + H + 2 * GN)            # x, z, dt, B, C
    writes = Dn * (2 if cfg["combine"] else 1)
    return Bt * L * (reads + writes) * e


def algorithmic_flops(cfg):
    """fp32 operations the definition needs per call, both directions: per (token, channel, direction)
    conv 4 fma (8), two SiLU (mul, exp, add, rcp, mul = 5 each), Delta*xc (1), D*xc fma (2), gate mul (1) = 22,
    plus per state: decay argument mul, exp, input mul, two fma = 7 (6 without a per-state decay: the exponential
    and its argument are then per token-channel)."""
    Bt, L, Dn, N = cfg["batch"], cfg["seqlen"], cfg["d_inner"], cfg["d_state"]
    per_state = 7 if cfg["a_kind"] == 0 else 5
    per_tc = 22 + per_state * N + (0 if cfg["a_kind"] == 0 else 2)
    return 2 * Bt * L * Dn * per_tc + (Bt * L * Dn if not cfg["combine"] else 0)


def algorithmic_flops_bwd(cfg):
    """fp32 operations the gradients of the selective-scan layout need per call, both directions, counting the forward
    quantities the backward rule uses (they have to be formed again): per (token, channel, direction) and state the
    forward's 7, then dh (fma 2), the dB and dC terms (2), dh*h_prev*a (2), its uses in dA (fma 2) and dDelta (fma 2),
    dh.B (fma 2), dh*a (1) and the two adds of the group sums (2) = 22; per (token, channel, direction) besides the
    forward's 22: SiLU' twice (6 each), dz, dy, dD (4), dDelta / dxc assembly (4), conv gradient (4 fma for dx, 4 for
    dw, 1 for db = 17), = 59."""
    Bt, L, Dn, N = cfg["batch"], cfg["seqlen"], cfg["d_inner"], cfg["d_state"]
    return 2 * Bt * L * Dn * (59 + 22 * N)


def algorithmic_bytes_bwd(cfg, shared_inputs=True):
    """Bytes the gradient call must move once: x, z, dt, dout read, dx, dz, ddt written per direction's activations
    (B, C and their fp32 gradients amortise over d_inner)."""
    e = 2 if cfg["io"] == "bf16" else 4
    Bt, L, Dn, GN = cfg["batch"], cfg["seqlen"], cfg["d_inner"], cfg["n_groups"] * cfg["d_state"]
    ndir = 1 if shared_inputs else 2
    out_w = Dn * (2 if cfg["combine"] else 1)
    return Bt * L * (ndir * (3 * Dn + 2 * GN) * e + out_w * e + ndir * (3 * Dn * e + 2 * GN * 4))


SSD_CHUNK = 64


def ssd_matrix_flops(cfg, chunk=SSD_CHUNK):
    """Matrix-core flops of the chunked form of the scalar-decay (Mamba-2) recurrence, both directions: per token and
    head 2*Q*P (masked scores times inputs) + 2*N*P (C times the carried state) + 2*N*P (state update), plus the score
    tile 2*Q*N per token and group."""
    Bt, L, Dn, N, H, G = cfg["batch"], cfg["seqlen"], cfg["d_inner"], cfg["d_state"], cfg["n_heads"], cfg["n_groups"]
    P = Dn // H
    per_token = H * (2 * chunk * P + 4 * N * P) + G * 2 * chunk * N
    return 2 * Bt * L * per_token
