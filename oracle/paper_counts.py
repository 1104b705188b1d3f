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
