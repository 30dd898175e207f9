"""Shape bookkeeping against the numbers the paper prints (App. C, Mamba-2 layer FLOP table)."""
import os

from paper_2511_15927_amd import shapes, synth


def golden():
    vals = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "flops_mamba_layer.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            vals[k] = float(v)
    return vals


def test_paper_layer_flops_reproduced():
    g = golden()
    # D_in = 2*d_inner (x, gate) + 2*d_state (B, C, one group) + n_heads (Delta) fixes 120 heads of width 32
    n_heads = int(g["D_in"]) - 2 * int(g["d_inner"]) - 2 * int(g["d_state"])
    assert n_heads == 120 and int(g["d_inner"]) // n_heads == 32
    assert shapes.in_proj_width(3840, 1, 128, n_heads) == g["D_in"]
    assert shapes.conv_channels(3840, 1, 128, 1) == g["conv_ch"]
    f = shapes.paper_flops_per_token(1920, 3840, 128, 4, n_heads)
    # the table prints millions with two decimals (three for the conv), truncated or rounded
    assert abs(f["in_proj"] / 1e6 - g["in_proj_M"]) < 0.01 and f["in_proj"] == 2 * 1920 * 8056
    assert abs(f["conv"] / 1e6 - g["conv_M"]) < 0.001 and f["conv"] == 4096 * 4
    assert abs(f["scan"] / 1e6 - g["scan_M"]) < 0.01 and f["scan"] == 2 * 3840 * 128
    assert abs(f["out_proj"] / 1e6 - g["out_proj_M"]) < 0.01 and f["out_proj"] == 2 * 3840 * 1920
    assert abs(f["one_direction"] / 1e6 - g["one_direction_M"]) < 0.01
    assert abs(f["bidirectional"] / 1e6 - g["bidirectional_M"]) < 0.011   # the table doubles the rounded subtotal


def test_algorithmic_bytes_and_flops_of_the_headline():
    cfg = synth.CONFIGS["headline"]
    tokens = cfg["batch"] * cfg["seqlen"]
    assert shapes.algorithmic_bytes(cfg) == tokens * (3 * 4096 + 2 * 16 + 4096) * 2     # 8 B per token-channel + B, C
    assert shapes.algorithmic_flops(cfg) == tokens * 4096 * (2 * (22 + 7 * 16) + 1)
    assert synth.conv_channels(synth.CONFIGS["paper_1p3b"]) == 4096
