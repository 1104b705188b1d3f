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


def test_step3_row_of_the_decoding_cost_table():
    """Section 4.2: max(core flop cost, cache byte cost) + linear flop cost, per 1M tokens, on the four
    accelerators of the unit-cost table; the printed Step-3 row has three decimals."""
    g = _golden()
    for ctx, tag in ((8192, "8k"), (32768, "32k")):
        for hw in ("H800", "H20", "A800", "910B"):
            cost = pc.step3_attention_cost_per_million_tokens(ctx, g["unit_cost_flop_" + hw], g["unit_cost_byte_" + hw])
            printed = g[f"attn_cost_{tag}_{hw}"]
            # half a unit of the last printed decimal, plus the rounding of the unit costs to three digits
            assert abs(cost - printed) <= 0.0005 + 0.004 * printed, (ctx, hw, cost)


def test_cost_formula_takes_the_larger_of_compute_and_memory():
    # memory-bound on H800 (cheap flops), compute-bound on H20 (cheap bytes) at 8K: Section 4.2's point
    g = _golden()
    L, H, D = int(g["layers"]), int(g["n_q_heads"]), int(g["head_dim"])
    fl, by = pc.attn_flops_per_decoded_token(L, H, D, 8192), pc.kv_bytes_per_decoded_token(L, D, 1, 8192)
    assert fl * g["unit_cost_flop_H800"] < by * g["unit_cost_byte_H800"]
    assert fl * g["unit_cost_flop_H20"] > by * g["unit_cost_byte_H20"]
    assert pc.attention_cost_per_token(fl, by, 0.0, 1.0, 0.0) == fl and pc.attention_cost_per_token(fl, by, 0.0, 0.0, 1.0) == by
    # a sum instead of a max, or a dropped linear term, misses the printed value
    bad_sum = 1e6 * (fl * g["unit_cost_flop_H20"] + by * g["unit_cost_byte_H20"]
                     + pc.attn_linear_flops_per_decoded_token(L, 7168, 2048, H, D) * g["unit_cost_flop_H20"])
    assert abs(bad_sum - g["attn_cost_8k_H20"]) > 0.005
    cf, cb = pc.unit_costs(3600.0, 1e15, 1e12)
    assert cf == 1e-15 and cb == 1e-12


def test_printed_rooflines_follow_from_the_printed_unit_costs():
    """Section 5.1 quotes the computation-bandwidth ratio of three accelerators; Section 4.2's unit costs give
    the same ratios (the hourly price cancels).  Two places of the paper that must agree, and do."""
    g = _golden()
    for hw in ("H20", "A800", "910B"):
        ratio = pc.ridge_point_from_unit_costs(g["unit_cost_flop_" + hw], g["unit_cost_byte_" + hw])
        assert abs(ratio - g["roofline_" + hw]) <= 0.01 * g["roofline_" + hw], (hw, ratio)
    cf, cb = pc.unit_costs(2.0, 1e15, 2e12)
    assert abs(pc.ridge_point_from_unit_costs(cf, cb) - pc.ridge_point(1e15, 2e12)) < 1e-9 * 500
    # MFA at 8 bits (128) sits below A800 and 910B and above H20, as the text says
    ai = pc.arithmetic_intensity(int(g["n_q_heads"]), int(g["head_dim"]), 1)
    assert g["roofline_H20"] < ai < g["roofline_A800"] < g["roofline_910B"]


def test_mi355x_column():
    """The extension by this build's accelerator: by the paper's own model MFA stays on the memory side of
    MI355X's ridge for every cache width and query-token count built here except 4-bit with four tokens."""
    col = pc.mi355x_column()
    assert col[(2, 1)][:2] == (64.0, 312.5) and col[(1, 1)][:2] == (128.0, 625.0) and col[(0.5, 1)][:2] == (256.0, 625.0)
    assert col[(1, 2)][0] == 256.0 and col[(0.5, 2)][0] == 512.0
    assert all(bound == "memory" for (w, n), (_, _, bound) in col.items() if (w, n) != (0.5, 4))
    assert col[(0.5, 4)][2] == "compute"
    # lower bound of the benchmark call: 64 x 4096 tokens, 1024 bytes and 4*64*256 flop per cached token
    t = pc.attention_time_bound(64 * 4096, 1024, 4 * 64 * 256, pc.MI355X["peak_flops_bf16"], pc.MI355X["peak_bytes_per_s"])
    assert abs(t - 33.554432e-6) < 1e-12
