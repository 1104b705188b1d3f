"""Pins for the oracle's 4-bit cache format (Section 5.2 discusses a cache kept in 4 bits and computed on in 8;
the format is this build's reading: OCP e2m1 elements, two per byte, one fp32 scale per token and tensor).
Checked against the format's definition typed out here, torch recipes, and the already pinned bf16 path."""
import numpy as np
import pytest
import torch

from paper_2507_19427_amd import workloads as W

# e2m1 as the OCP microscaling formats specification lists it: codes 0..7, then the same with the sign bit
E2M1_MAGNITUDES = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def test_all_sixteen_codes_decode_to_the_listed_values(oracle):
    for c in range(16):
        want = E2M1_MAGNITUDES[c & 7] * (-1.0 if c & 8 else 1.0)
        got = oracle.decode_e2m1(c)
        assert got == want and np.signbit(got) == bool(c & 8), (c, got)


def _encode_via_quantiser(oracle, values):
    """A row that contains 6 has scale exactly 1, so the quantiser reduces to the bare encoder.  The row is
    [6, 0, values...] padded to an even length; returns one code per value."""
    vals = list(np.asarray(values, dtype=np.float32))
    row = np.array([6.0, 0.0] + vals + ([0.0] if len(vals) % 2 else []), dtype=np.float32)[None, :]
    packed, scales = oracle.quantize_rows_e2m1(row)
    assert scales[0] == np.float32(1.0)
    assert packed[0, 0] == 0x07                     # 6 in the low four bits, 0 above it
    codes = np.stack([packed[0] & 15, packed[0] >> 4], axis=1).reshape(-1)
    return codes[2:2 + len(vals)]


def test_every_code_encodes_to_itself(oracle):
    vals = [oracle.decode_e2m1(c) for c in range(16)]
    got = _encode_via_quantiser(oracle, vals)
    assert list(got) == list(range(16))             # -0.0 keeps its sign bit: code 8


def test_midpoints_go_to_the_even_code_and_neighbours_to_the_nearest(oracle):
    for lo in range(7):
        a, b = E2M1_MAGNITUDES[lo], E2M1_MAGNITUDES[lo + 1]
        mid = np.float32(0.5 * (a + b))
        even = lo if lo % 2 == 0 else lo + 1
        below, above = np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(9))
        got = _encode_via_quantiser(oracle, [mid, below, above, -mid, -below, -above])
        assert list(got) == [even, lo, lo + 1, even | 8, lo | 8, (lo + 1) | 8], (a, b, list(got))


def test_packing_puts_the_even_element_in_the_low_bits(oracle):
    row = np.array([[6.0, -0.5, 1.0, 3.0]], dtype=np.float32)
    packed, _ = oracle.quantize_rows_e2m1(row)
    assert list(packed[0]) == [0x7 | (0x9 << 4), 0x2 | (0x5 << 4)]


def test_quantiser_matches_the_generator_recipe_in_torch(oracle):
    g = torch.Generator().manual_seed(21)
    x = torch.randn(400, 256, generator=g) * (torch.rand(400, 1, generator=g) * 20 + 1e-3)
    x[3] = 0.0
    x[4, ::2] = -0.0
    p_ref, s_ref = W.quantize_e2m1_per_token(x)
    packed, scales = oracle.quantize_rows_e2m1(x.numpy())
    assert np.array_equal(scales, s_ref.numpy())
    assert np.array_equal(packed, p_ref.numpy())
    # the largest element of a row above the floor always lands on +-6
    codes = np.stack([packed & 15, packed >> 4], axis=2).reshape(400, 256)
    idx = np.abs(x.numpy()).argmax(axis=1)
    rows = np.arange(400) != 3
    assert ((codes[np.arange(400), idx] & 7)[rows] == 7).all()


def test_dequantised_value_is_within_half_a_step(oracle):
    g = torch.Generator().manual_seed(22)
    x = (torch.randn(100, 64, generator=g) * 3).numpy().astype(np.float32)
    packed, scales = oracle.quantize_rows_e2m1(x)
    codes = np.stack([packed & 15, packed >> 4], axis=2).reshape(100, 64)
    dec = np.vectorize(oracle.decode_e2m1)(codes)
    mag = np.abs(dec)
    step = np.where(mag < 2.0, 0.5, np.where(mag < 4.0, 1.0, 2.0))
    err = np.abs(dec - x.astype(np.float64) / scales.astype(np.float64)[:, None])
    assert (err <= 0.5 * step * (1 + 1e-6)).all()


def _dequantised_bf16(packed, scales):
    """Exact when the scales are powers of two: an e2m1 value has two significant bits."""
    codes = torch.stack([packed & 15, packed >> 4], dim=-1).reshape(*packed.shape[:-1], -1)
    table = torch.tensor(E2M1_MAGNITUDES + [-m for m in E2M1_MAGNITUDES], dtype=torch.float64)
    vals = table[codes.long()] * scales.double().unsqueeze(-1)
    out = vals.to(torch.bfloat16)
    assert torch.equal(out.double(), vals)
    return out


def test_attention_over_the_4bit_cache_equals_attention_over_its_dequantised_values(oracle):
    """With power-of-two scales code*scale is a bf16 number, so the bf16 path (pinned by brute force elsewhere)
    must give the same result: pins the byte/nibble indexing and the use of the scales."""
    g = torch.Generator().manual_seed(23)
    B, H, D, S = 3, 4, 32, 19
    q = torch.randn(B, H, D, generator=g).to(torch.bfloat16)
    k = torch.randint(0, 256, (B, S, D // 2), generator=g, dtype=torch.uint8)
    v = torch.randint(0, 256, (B, S, D // 2), generator=g, dtype=torch.uint8)
    ks = torch.pow(2.0, torch.randint(-3, 3, (B, S), generator=g).float())
    vs = torch.pow(2.0, torch.randint(-3, 3, (B, S), generator=g).float())
    lens = np.array([19, 1, 7], dtype=np.int32)
    got = oracle.decode_attn(oracle.bits_of(q), k.numpy(), v.numpy(), lens, 0.25, k_scale=ks.numpy(), v_scale=vs.numpy(),
                             kv_dtype=oracle.KV_E2M1)
    ref = oracle.decode_attn(oracle.bits_of(q), oracle.bits_of(_dequantised_bf16(k, ks)), oracle.bits_of(_dequantised_bf16(v, vs)),
                             lens, 0.25)
    assert np.array_equal(got, ref)


def test_attention_over_the_4bit_cache_brute_force(oracle):
    case = W.make_contiguous_case("fp4brute", 24, B=2, S=11, seq_lens=[11, 4], kv_dtype="fp4", poison=True, H=3, D=16)
    got = oracle.decode_attn(oracle.bits_of(case.q), case.k.numpy(), case.v.numpy(), case.seq_lens.numpy(), case.scale,
                             k_scale=case.k_scale.numpy(), v_scale=case.v_scale.numpy(), kv_dtype=oracle.KV_E2M1)
    table = np.array(E2M1_MAGNITUDES + [-m for m in E2M1_MAGNITUDES])
    for b, L in enumerate([11, 4]):
        def deq(packed, scales):
            codes = np.stack([packed & 15, packed >> 4], axis=-1).reshape(packed.shape[0], -1)
            return table[codes] * scales.astype(np.float64)[:, None]
        K = deq(case.k[b, :L].numpy(), case.k_scale[b, :L].numpy())
        V = deq(case.v[b, :L].numpy(), case.v_scale[b, :L].numpy())
        for h in range(3):
            s = case.scale * (K @ case.q[b, h].double().numpy())
            p = np.exp(s - s.max())
            ref = (p / p.sum()) @ V
            assert np.abs(got[b, h] - ref).max() <= 1e-6 * max(1.0, np.abs(ref).max())


def test_paged_4bit_cache_equals_contiguous(oracle):
    case = W.make_paged_case("fp4paged", 25, [70, 1, 0, 64, 129], kv_dtype="fp4", spare_pages=3, poison=True, H=2, D=16)
    contig = W.paged_to_contiguous(case, poison=True)
    a = oracle.decode_attn_paged(oracle.bits_of(case.q), case.k_pool.numpy(), case.v_pool.numpy(), case.block_table.numpy(),
                                 case.seq_lens.numpy(), case.scale, k_scale_pool=case.k_scale_pool.numpy(),
                                 v_scale_pool=case.v_scale_pool.numpy(), kv_dtype=oracle.KV_E2M1)
    b = oracle.decode_attn(oracle.bits_of(contig.q), contig.k.numpy(), contig.v.numpy(), contig.seq_lens.numpy(), contig.scale,
                           k_scale=contig.k_scale.numpy(), v_scale=contig.v_scale.numpy(), kv_dtype=oracle.KV_E2M1)
    assert np.array_equal(a, b)
    assert np.isfinite(a).all() and (a[2] == 0).all()
