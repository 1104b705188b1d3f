"""Shape pins: the oracle's accounting functions must reproduce the figures the paper prints
for its own model (tests/golden/paper_counts.txt lists each with its place in the paper)."""
import os

from oracle import paper_counts as pc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_counts.txt")


def _golden():
    vals = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    return vals


def _matches_printed(value, printed, digits=3):
    """True if value rounds to the printed figure at the printed number of significant digits."""
    return float(f"{value:.{digits - 1}e}") == float(f"{printed:.{digits - 1}e}")


def test_step3_rows_of_the_decoding_tables():
    g = _golden()
    L, Hd, r = int(g["layers"]), int(g["hidden"]), int(g["q_rank"])
    H, D = int(g["n_q_heads"]), int(g["head_dim"])
    assert pc.kv_bytes_per_token_per_layer(D, 1) == g["kv_bytes_per_token_per_layer"]
    assert _matches_printed(pc.kv_bytes_per_decoded_token(L, D, 1, 8192), g["kv_bytes_per_token_8k"])
    assert _matches_printed(pc.kv_bytes_per_decoded_token(L, D, 1, 32768), g["kv_bytes_per_token_32k"])
    assert _matches_printed(pc.attn_flops_per_decoded_token(L, H, D, 8192), g["attn_flops_per_token_8k"])
    assert _matches_printed(pc.attn_flops_per_decoded_token(L, H, D, 32768), g["attn_flops_per_token_32k"])
    assert _matches_printed(pc.attn_linear_flops_per_decoded_token(L, Hd, r, H, D), g["linear_flops_per_token"])
    assert pc.arithmetic_intensity(H, D, 1) == g["arithmetic_intensity_8bit"]
    mb = pc.attn_linear_weight_bytes_per_gpu(Hd, r, H, D, 1, 8) / 1e6
    assert round(mb) == g["linear_weight_mb_per_gpu"]


def test_wrong_shapes_miss_the_printed_figures():
    """A plausible misreading (two KV heads, head dim 128, 32 heads) must not reproduce the table."""
    g = _golden()
    L = int(g["layers"])
    assert not _matches_printed(L * 8192 * pc.kv_bytes_per_token_per_layer(256, 1, 2, 2), g["kv_bytes_per_token_8k"])
    assert not _matches_printed(pc.kv_bytes_per_decoded_token(L, 128, 1, 8192), g["kv_bytes_per_token_8k"])
    assert not _matches_printed(pc.attn_flops_per_decoded_token(L, 32, 256, 8192), g["attn_flops_per_token_8k"])
    assert pc.arithmetic_intensity(64, 256, 2) == 64     # bf16 cache halves the intensity
