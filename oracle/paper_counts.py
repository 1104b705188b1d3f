"""Byte and flop accounting of one decoded token, written out from the model shape.

Test infrastructure (part of the oracle): the paper prints these counts for
its model (Section 4.1, tables of per-token memory access and computation at
8K and 32K context; Section 5.1, arithmetic intensity; Section 6, bytes per
cached token and linear-weight bytes).  Reproducing the printed figures from
(layers, heads, head dim, hidden size, query rank) pins the shapes the
attention oracle and the GPU kernels assume: one key head and one value head
of the query head dimension, 64 query heads, rank-2048 query factorisation.
"""


def kv_bytes_per_token_per_layer(head_dim, bytes_per_elem, n_k_heads=1, n_v_heads=1):
    """Cache record of one token in one layer: one key row + one value row."""
    return (n_k_heads + n_v_heads) * head_dim * bytes_per_elem


def kv_bytes_per_decoded_token(layers, head_dim, bytes_per_elem, ctx):
    """Cache bytes read to decode one token at context length ctx (all layers)."""
    return layers * ctx * kv_bytes_per_token_per_layer(head_dim, bytes_per_elem)


def attn_flops_per_decoded_token(layers, n_q_heads, head_dim, ctx):
    """Scores (2*H*D per cached token) plus weighted sum (2*H*D), all layers, no linears."""
    return layers * ctx * 4 * n_q_heads * head_dim


def attn_linear_flops_per_decoded_token(layers, d_model, q_rank, n_q_heads, head_dim):
    """Linears around attention: W_qa, W_qb, key and value projection, output projection."""
    macs = (d_model * q_rank + q_rank * n_q_heads * head_dim
            + 2 * d_model * head_dim + n_q_heads * head_dim * d_model)
    return 2 * layers * macs


def attn_linear_weight_bytes_per_gpu(d_model, q_rank, n_q_heads, head_dim, bytes_per_elem, o_proj_tp):
    """Linear weights one GPU streams per layer: everything replicated except the output
    projection, which is sharded o_proj_tp ways (Section 6, footnote)."""
    elems = (d_model * q_rank + q_rank * n_q_heads * head_dim + 2 * d_model * head_dim
             + n_q_heads * head_dim * d_model // o_proj_tp)
    return elems * bytes_per_elem


def arithmetic_intensity(n_q_heads, head_dim, bytes_per_elem):
    """Attention flops per cache byte: 4*H*D flop over 2*D*bytes per cached token."""
    return 4 * n_q_heads * head_dim / kv_bytes_per_token_per_layer(head_dim, bytes_per_elem)


# ---------------------------------------------------------------------------
# The paper's theoretical decoding cost of the attention part (Section 4.2):
# the larger of the core's computation cost and its cache-access cost, plus the
# computation cost of the linears before and after, each priced by the
# accelerator's cost per flop and per byte of memory access.
# ---------------------------------------------------------------------------

def unit_costs(price_per_hour, peak_flops, peak_bytes_per_s):
    """(cost per flop, cost per byte) of an accelerator rented at price_per_hour and fully used."""
    per_second = price_per_hour / 3600.0
    return per_second / peak_flops, per_second / peak_bytes_per_s


def attention_cost_per_token(attn_flops, kv_bytes, linear_flops, cost_per_flop, cost_per_byte):
    """max(flop cost of the attention core, byte cost of its cache reads) + flop cost of the linears."""
    return max(attn_flops * cost_per_flop, kv_bytes * cost_per_byte) + linear_flops * cost_per_flop


def step3_attention_cost_per_million_tokens(ctx, cost_per_flop, cost_per_byte, layers=61, n_q_heads=64, head_dim=256,
                                            d_model=7168, q_rank=2048, kv_bytes_per_elem=1):
    """The Step-3 row of the paper's decoding-cost table, from the model shape (8-bit cache)."""
    per_token = attention_cost_per_token(
        attn_flops_per_decoded_token(layers, n_q_heads, head_dim, ctx),
        kv_bytes_per_decoded_token(layers, head_dim, kv_bytes_per_elem, ctx),
        attn_linear_flops_per_decoded_token(layers, d_model, q_rank, n_q_heads, head_dim),
        cost_per_flop, cost_per_byte)
    return 1e6 * per_token



# ---------------------------------------------------------------------------
# Roofline of an accelerator as the paper uses the word (Section 5.1): peak
# computation over peak memory bandwidth, in flop per byte.  An attention design
# whose arithmetic intensity is below it is bound by memory, above it by compute.
# ---------------------------------------------------------------------------

def ridge_point(peak_flops, peak_bytes_per_s):
    return peak_flops / peak_bytes_per_s


def ridge_point_from_unit_costs(cost_per_flop, cost_per_byte):
    """The same ratio from the paper's unit-cost table: the hourly price cancels."""
    return cost_per_byte / cost_per_flop


def attention_time_bound(kv_tokens, bytes_per_kv_token, flops_per_kv_token, peak_flops, peak_bytes_per_s):
    """Lower bound (seconds) on one attention call that reads kv_tokens cached tokens: the larger of
    its memory time and its compute time at the accelerator's peaks."""
    return max(kv_tokens * bytes_per_kv_token / peak_bytes_per_s, kv_tokens * flops_per_kv_token / peak_flops)


# The accelerator this build runs on, by its published dense peaks (no price is asserted, so no cost
# column follows from it): the extension of the paper's accelerator table by one column.
MI355X = {"peak_flops_bf16": 2.5e15, "peak_flops_8bit": 5.0e15, "peak_bytes_per_s": 8.0e12}


def mi355x_column(n_q_heads=64, head_dim=256):
    """Where MFA's arithmetic intensity sits against MI355X, for the cache widths and query-token
    counts this build supports: {(bytes per element, query tokens): (intensity, ridge, bound)}."""
    out = {}
    for bytes_per_elem, peak in ((2, MI355X["peak_flops_bf16"]), (1, MI355X["peak_flops_8bit"]), (0.5, MI355X["peak_flops_8bit"])):
        ridge = ridge_point(peak, MI355X["peak_bytes_per_s"])
        for q_tokens in (1, 2, 4):
            ai = q_tokens * arithmetic_intensity(n_q_heads, head_dim, bytes_per_elem)
            out[(bytes_per_elem, q_tokens)] = (ai, ridge, "memory" if ai < ridge else "compute")
    return out
