"""Pins for the attention oracle against things other than itself: brute force, closed forms,
invariants of softmax attention, and torch's fp64 scaled_dot_product_attention."""
import math

import numpy as np
import pytest
import torch

from paper_2507_19427_amd import workloads as W

SCALE = 1.0 / 16.0


def _bits(oracle, case):
    b = oracle.bits_of
    return dict(q=b(case.q), k=b(case.k), v=b(case.v),
                k_scale=None if case.k_scale is None else b(case.k_scale),
                v_scale=None if case.v_scale is None else b(case.v_scale),
                kv_dtype=oracle.KV_E4M3 if case.kv_dtype == "fp8" else oracle.KV_BF16)


def _run(oracle, case, **kw):
    a = _bits(oracle, case)
    return oracle.decode_attn(a["q"], a["k"], a["v"], case.seq_lens.numpy(), case.scale,
                              k_scale=a["k_scale"], v_scale=a["v_scale"], kv_dtype=a["kv_dtype"], **kw)


def _dequant(case):
    """K, V as float64 arrays via torch's casts (library routine, not the oracle's decoders)."""
    k = case.k.to(torch.float64)
    v = case.v.to(torch.float64)
    if case.kv_dtype == "fp8":
        k = k * case.k_scale.to(torch.float64).unsqueeze(-1)
        v = v * case.v_scale.to(torch.float64).unsqueeze(-1)
    return k.numpy(), v.numpy()


def _brute(case):
    q = case.q.to(torch.float64).numpy()
    k, v = _dequant(case)
    B, H, D = q.shape
    out = np.zeros((B, H, D))
    for b in range(B):
        L = int(case.seq_lens[b])
        if L == 0:
            continue
        for h in range(H):
            w = np.array([math.exp(case.scale * float(np.dot(q[b, h], k[b, j]))) for j in range(L)])
            out[b, h] = (w[:, None] * v[b, :L]).sum(0) / w.sum()
    return out


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_brute_force_tiny(oracle, kv_dtype):
    case = W.make_contiguous_case("t", 11, B=3, S=37, seq_lens=[37, 1, 20], kv_dtype=kv_dtype, H=5, D=16,
                                  scale=0.25)
    got = _run(oracle, case)
    ref = _brute(case)
    assert np.abs(got - ref).max() <= 1e-6 * np.abs(ref).max()     # fp32 output rounding only
    assert np.abs(got - ref.astype(np.float32)).max() <= 2e-7


def test_two_token_closed_form(oracle):
    """q = e0*a: weights are a logistic function of scale*a*(k0-k1)[0]."""
    H, D = 1, 8
    q = torch.zeros(1, H, D)
    q[0, 0, 0] = 3.0
    k = torch.zeros(1, 2, D)
    k[0, 0, 0], k[0, 1, 0] = 2.0, -1.0
    v = torch.zeros(1, 2, D)
    v[0, 0, :], v[0, 1, :] = 1.0, -3.0
    got = oracle.decode_attn(oracle.bits_of(q.bfloat16()), oracle.bits_of(k.bfloat16()),
                             oracle.bits_of(v.bfloat16()), [2], 0.5)
    w0 = 1.0 / (1.0 + math.exp(-0.5 * 3.0 * 3.0))
    want = w0 * 1.0 + (1 - w0) * -3.0
    assert np.allclose(got[0, 0], np.float32(want), rtol=0, atol=1e-7)


def test_weights_sum_to_one_and_reproduce_output(oracle):
    case = W.make_contiguous_case("t", 12, B=2, S=300, seq_lens=[300, 123], H=4, D=32)
    a = _bits(oracle, case)
    k, v = _dequant(case)
    for b, h in [(0, 0), (1, 3)]:
        w, row = oracle.attn_weights(a["q"], a["k"], a["v"], case.seq_lens.numpy(), case.scale, b, h)
        assert abs(w.sum() - 1.0) <= 1e-14 and (w >= 0).all()
        assert np.allclose(row, (w[:, None] * v[b, :len(w)]).sum(0), rtol=0, atol=1e-6)


def test_context_length_one_returns_value_row(oracle):
    case = W.make_contiguous_case("t", 13, B=4, S=8, seq_lens=[1, 1, 1, 1], H=6, D=32)
    got = _run(oracle, case)
    v = case.v.to(torch.float32).numpy()
    for b in range(4):
        for h in range(6):
            assert np.array_equal(got[b, h], v[b, 0])


def test_empty_context_gives_zero(oracle):
    case = W.make_contiguous_case("t", 14, B=2, S=8, seq_lens=[0, 5], H=3, D=16)
    got = _run(oracle, case)
    assert np.array_equal(got[0], np.zeros((3, 16), np.float32)) and np.isfinite(got).all()


def test_zero_query_returns_mean_value(oracle):
    case = W.make_contiguous_case("t", 15, B=2, S=50, seq_lens=[50, 17], H=2, D=16)
    case.q.zero_()
    got = _run(oracle, case)
    _, v = _dequant(case)
    for b, L in enumerate([50, 17]):
        assert np.allclose(got[b, 0], v[b, :L].mean(0), rtol=0, atol=1e-7)


def test_identical_keys_return_mean_value(oracle):
    case = W.make_contiguous_case("t", 16, B=1, S=40, H=3, D=16)
    case.k[:] = case.k[:, :1]
    got = _run(oracle, case)
    _, v = _dequant(case)
    assert np.allclose(got[0], np.broadcast_to(v[0].mean(0), (3, 16)), rtol=0, atol=1e-7)


def test_dominant_key_selects_its_value_row(oracle):
    case = W.make_contiguous_case("t", 17, B=1, S=30, H=1, D=16, scale=1.0)
    case.q.zero_()
    case.q[0, 0, 0] = 1.0
    case.k.zero_()
    case.k[0, 7, 0] = 64.0          # score 64 above all the others: leakage < e^-64
    got = _run(oracle, case)
    assert np.array_equal(got[0, 0], case.v[0, 7].to(torch.float32).numpy())


def test_key_shift_invariance(oracle):
    """Adding one vector to every key adds the same constant to every score of a head."""
    case = W.make_contiguous_case("t", 18, B=1, S=64, H=4, D=16)
    # keep values exactly representable after the shift: small integers / 8
    case.k = (torch.round(case.k.float() * 8) / 8).bfloat16()
    base = _run(oracle, case)
    shifted = W.make_contiguous_case("t", 18, B=1, S=64, H=4, D=16)
    delta = torch.arange(16, dtype=torch.float32) / 8 - 1.0
    shifted.k = (case.k.float() + delta).bfloat16()
    assert torch.equal(shifted.k.float(), case.k.float() + delta)   # shift is exact in bf16
    got = _run(oracle, shifted)
    assert np.abs(got - base).max() <= 1e-6


def test_token_permutation_invariance(oracle):
    case = W.make_contiguous_case("t", 19, B=2, S=90, seq_lens=[90, 90], H=3, D=32)
    base = _run(oracle, case)
    perm = torch.randperm(90, generator=torch.Generator().manual_seed(0))
    case.k = case.k[:, perm].contiguous()
    case.v = case.v[:, perm].contiguous()
    got = _run(oracle, case)
    assert np.abs(got - base).max() <= 1e-6


def test_output_is_convex_combination(oracle):
    case = W.make_contiguous_case("t", 20, B=2, S=70, seq_lens=[70, 33], H=4, D=16)
    got = _run(oracle, case)
    _, v = _dequant(case)
    for b, L in enumerate([70, 33]):
        assert (got[b] <= v[b, :L].max(0) + 1e-6).all() and (got[b] >= v[b, :L].min(0) - 1e-6).all()


def test_split_merge_identity(oracle):
    """Attention over [0,L) equals the log-sum-exp merge of attention over [0,a) and [a,L)."""
    case = W.make_contiguous_case("t", 21, B=1, S=200, H=4, D=32, poison=False)
    full, lse = _run(oracle, case, return_lse=True)
    for a_ in (1, 77, 199):
        left = W.make_contiguous_case("t", 21, B=1, S=200, seq_lens=[a_], H=4, D=32, poison=False)
        o1, l1 = _run(oracle, left, return_lse=True)
        right = W.make_contiguous_case("t", 21, B=1, S=200, H=4, D=32, poison=False)
        right.k = right.k[:, a_:].contiguous()
        right.v = right.v[:, a_:].contiguous()
        right.seq_lens = torch.tensor([200 - a_], dtype=torch.int32)
        o2, l2 = _run(oracle, right, return_lse=True)
        m = np.maximum(l1, l2)
        w1, w2 = np.exp(l1 - m), np.exp(l2 - m)
        merged = (w1[..., None] * o1 + w2[..., None] * o2) / (w1 + w2)[..., None]
        assert np.abs(merged - full).max() <= 1e-6
        assert np.abs(m + np.log(w1 + w2) - lse).max() <= 1e-12


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_against_torch_sdpa_fp64(oracle, kv_dtype):
    case = W.make_contiguous_case("t", 22, B=2, S=256, kv_dtype=kv_dtype, H=8, D=64, scale=0.125)
    got = _run(oracle, case)
    k, v = _dequant(case)
    B, H, D = case.q.shape
    kk = torch.from_numpy(k)[:, None].expand(B, H, 256, D)
    vv = torch.from_numpy(v)[:, None].expand(B, H, 256, D)
    ref = torch.nn.functional.scaled_dot_product_attention(case.q.double()[:, :, None, :], kk, vv,
                                                           scale=0.125)[:, :, 0].numpy()
    assert np.abs(got - ref).max() <= 1e-6


def test_config1_against_torch_sdpa_fp64(oracle):
    """The tiny named workload at its real shape (64 heads, dim 256, context 256)."""
    case = W.config1_tiny()
    got = _run(oracle, case)
    B, H, D = case.q.shape
    kk = case.k.double()[:, None].expand(B, H, 256, D)
    vv = case.v.double()[:, None].expand(B, H, 256, D)
    ref = torch.nn.functional.scaled_dot_product_attention(case.q.double()[:, :, None, :], kk, vv,
                                                           scale=SCALE)[:, :, 0].numpy()
    assert got.shape == (2, 64, 256) and got.dtype == np.float32
    assert np.abs(got - ref).max() <= 1e-6


def test_fp8_unit_scale_equals_bf16_on_representable_values(oracle):
    """With scale 1 and values that e4m3 holds exactly, the fp8 path must equal the bf16 path bitwise."""
    g = torch.Generator().manual_seed(23)
    B, S, H, D = 2, 48, 4, 32
    codes_k = torch.randint(0, 0x7F, (B, S, D), generator=g, dtype=torch.int32).to(torch.uint8)
    codes_v = torch.randint(0, 0x7F, (B, S, D), generator=g, dtype=torch.int32).to(torch.uint8)
    sign = torch.randint(0, 2, (B, S, D), generator=g, dtype=torch.int32).to(torch.uint8) * 0x80
    k8 = ((codes_k % 0x60) | sign).view(torch.float8_e4m3fn)     # |value| <= 28: keeps scores moderate
    v8 = (codes_v | sign).view(torch.float8_e4m3fn)
    q = (torch.randn(B, H, D, generator=g) * 0.1).bfloat16()
    ones = np.ones((B, S), np.float32)
    lens = [S, 31]
    o8 = oracle.decode_attn(oracle.bits_of(q), oracle.bits_of(k8), oracle.bits_of(v8), lens, SCALE,
                            k_scale=ones, v_scale=ones, kv_dtype=oracle.KV_E4M3)
    o16 = oracle.decode_attn(oracle.bits_of(q), oracle.bits_of(k8.to(torch.bfloat16)),
                             oracle.bits_of(v8.to(torch.bfloat16)), lens, SCALE)
    assert np.array_equal(o8, o16)


def test_fp8_scales_are_applied_per_token(oracle):
    """Doubling every key scale equals doubling the softmax scale; doubling value scales doubles the output."""
    case = W.make_contiguous_case("t", 24, B=2, S=60, seq_lens=[60, 44], kv_dtype="fp8", H=4, D=32, poison=False)
    a = _bits(oracle, case)
    lens = case.seq_lens.numpy()
    base = oracle.decode_attn(a["q"], a["k"], a["v"], lens, 2 * SCALE, k_scale=a["k_scale"],
                              v_scale=a["v_scale"], kv_dtype=oracle.KV_E4M3)
    k2 = oracle.decode_attn(a["q"], a["k"], a["v"], lens, SCALE, k_scale=2 * a["k_scale"],
                            v_scale=a["v_scale"], kv_dtype=oracle.KV_E4M3)
    assert np.array_equal(base, k2)
    v2 = oracle.decode_attn(a["q"], a["k"], a["v"], lens, 2 * SCALE, k_scale=a["k_scale"],
                            v_scale=2 * a["v_scale"], kv_dtype=oracle.KV_E4M3)
    assert np.array_equal(v2, 2 * base)
    # scales really are per token: changing one token's scales must change the result
    ks = a["k_scale"].copy()
    ks[0, 5] *= 3
    assert not np.array_equal(base[0], oracle.decode_attn(a["q"], a["k"], a["v"], lens, 2 * SCALE, k_scale=ks,
                                                          v_scale=a["v_scale"], kv_dtype=oracle.KV_E4M3)[0])


def test_poisoned_tail_is_never_read(oracle):
    clean = W.make_contiguous_case("t", 25, B=2, S=40, seq_lens=[13, 40], H=2, D=16, poison=False)
    dirty = W.make_contiguous_case("t", 25, B=2, S=40, seq_lens=[13, 40], H=2, D=16, poison=True)
    assert torch.isnan(dirty.k[0, 13:].float()).all()
    assert np.array_equal(_run(oracle, clean), _run(oracle, dirty))


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_permuted_pages_equal_contiguous_bitwise(oracle, kv_dtype):
    lens = [1, 64, 65, 200, 0, 127]
    case = W.make_paged_case("p", 26, lens, kv_dtype=kv_dtype, spare_pages=5, H=4, D=32)
    contig = W.paged_to_contiguous(case)
    b = oracle.bits_of
    kd = oracle.KV_E4M3 if kv_dtype == "fp8" else oracle.KV_BF16
    sp = (None, None) if kv_dtype == "bf16" else (b(case.k_scale_pool), b(case.v_scale_pool))
    got, lse_p = oracle.decode_attn_paged(b(case.q), b(case.k_pool), b(case.v_pool), case.block_table.numpy(),
                                          case.seq_lens.numpy(), case.scale, k_scale_pool=sp[0],
                                          v_scale_pool=sp[1], kv_dtype=kd, return_lse=True)
    ref, lse_c = _run(oracle, contig, return_lse=True)
    assert np.array_equal(got, ref) and np.array_equal(lse_p, lse_c)
    assert np.isfinite(got).all()
    # the table really is permuted (not the identity layout)
    ids = case.block_table[case.block_table >= 0]
    assert not torch.equal(ids, torch.arange(len(ids), dtype=torch.int32))


def test_row_subset_matches_full(oracle):
    case = W.make_contiguous_case("t", 27, B=3, S=50, seq_lens=[50, 9, 30], H=4, D=16)
    full = _run(oracle, case)
    rows = [(2, 3), (0, 0), (1, 2)]
    sub = _run(oracle, case, rows=rows)
    for i, (bb, hh) in enumerate(rows):
        assert np.array_equal(sub[i], full[bb, hh])


@pytest.mark.parametrize("q_len", [2, 3, 4])
def test_several_query_tokens_equal_causal_attention_over_the_new_tokens(oracle, q_len):
    """A decode step with q_len new tokens per sequence (Section 5.2, multi-token prediction) is checked on the
    GPU against the single-token oracle called once per token with the length L - (q_len - 1 - j).  That
    composition is pinned here against torch's fp64 scaled_dot_product_attention with a mask that is causal
    among the last q_len positions, and against ragged lengths including L < q_len."""
    lens = [40, 1, 2, 3, 17, 0]
    case = W.make_contiguous_case("mt", 33 + q_len, B=len(lens), S=40, seq_lens=lens, poison=False, H=4, D=32, scale=0.2)
    qm = W.make_multi_query(case, q_len, 34)
    B, H, D = case.q.shape
    k, v = _dequant(case)
    for b, L in enumerate(lens):
        for j in range(q_len):
            Lj = max(L - (q_len - 1 - j), 0)
            sub = W.AttnCase(name="s", q=qm[b:b + 1, j].contiguous(), seq_lens=torch.tensor([Lj], dtype=torch.int32),
                             kv_dtype="bf16", k=case.k[b:b + 1], v=case.v[b:b + 1], scale=case.scale)
            got = _run(oracle, sub)[0]
            if Lj == 0:
                assert (got == 0).all()
                continue
            # rows of the mask: query token j sees positions < L - (q_len - 1 - j)
            kk = torch.from_numpy(k[b, :L])[None, None].expand(1, H, L, D)
            vv = torch.from_numpy(v[b, :L])[None, None].expand(1, H, L, D)
            mask = torch.zeros(q_len, L, dtype=torch.bool)
            for jj in range(q_len):
                mask[jj, :max(L - (q_len - 1 - jj), 0)] = True
            qq = qm[b].double().permute(1, 0, 2)[None]                      # [1, H, q_len, D]
            ref = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, attn_mask=mask[None, None], scale=0.2)
            assert np.abs(got - ref[0, :, j].numpy()).max() <= 1e-6
