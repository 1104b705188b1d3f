"""Pins for the oracle's linear maps and cache quantiser (the pieces around the attention core that the
attention layer of Section 6 counts: key/value projection of the new token, its 8-bit cache record, the
output projection).  Each check is against something other than the oracle itself: torch's CPU casts and
fp64 matmul, closed forms, or the format's own definition."""
import numpy as np
import pytest
import torch

from paper_2507_19427_amd import workloads as W


def _finite_e4m3_values(oracle):
    codes = [c for c in range(256) if (c & 0x7F) != 0x7F]
    return codes, np.array([oracle.decode_e4m3fn(c) for c in codes], dtype=np.float64)


def _encode_via_quantiser(oracle, values):
    """Rows that contain 448 have scale exactly 1, so the quantiser reduces to the bare encoder."""
    row = np.concatenate([[448.0], np.asarray(values, dtype=np.float32)]).astype(np.float32)[None, :]
    codes, scales = oracle.quantize_rows_e4m3(row)
    assert scales[0] == np.float32(1.0)
    return codes[0, 1:]


def test_every_finite_code_encodes_to_itself(oracle):
    codes, vals = _finite_e4m3_values(oracle)
    got = _encode_via_quantiser(oracle, vals)
    for c, g, v in zip(codes, got, vals):
        if v == 0.0:
            assert (g & 0x7F) == 0                      # +0 and -0 keep a zero magnitude
        else:
            assert g == c, (hex(c), hex(g), v)


def test_midpoints_round_to_the_even_code_and_neighbours_to_the_nearest(oracle):
    codes, vals = _finite_e4m3_values(oracle)
    pos = sorted((v, c) for c, v in zip(codes, vals) if c < 0x80)
    for (lo, clo), (hi, chi) in zip(pos[:-1], pos[1:]):
        mid = np.float32(0.5 * (lo + hi))
        assert float(mid) == 0.5 * (lo + hi)            # exactly representable in fp32
        even = clo if (clo & 1) == 0 else chi
        below = np.nextafter(mid, np.float32(0.0))
        above = np.nextafter(mid, np.float32(1e9))
        got = _encode_via_quantiser(oracle, [mid, below, above, -mid, -below, -above])
        assert list(got) == [even, clo, chi, even | 0x80, clo | 0x80, chi | 0x80], (lo, hi, list(map(hex, got)))


def test_encoder_matches_torch_cast_on_random_values(oracle):
    g = torch.Generator().manual_seed(11)
    x = torch.cat([torch.randn(4000, generator=g) * 100, torch.randn(4000, generator=g), torch.randn(4000, generator=g) * 0.01,
                   torch.rand(2000, generator=g) * 2 ** -6]).clamp_(-448, 448)
    want = x.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = _encode_via_quantiser(oracle, x.numpy())
    assert np.array_equal(got, want)


def test_saturation_and_quotient_clamp(oracle):
    # a row whose largest element is below the 1e-12 floor: scale = 1e-12/448, quotients stay small
    row = np.full((1, 8), 1e-20, dtype=np.float32)
    codes, scales = oracle.quantize_rows_e4m3(row)
    assert scales[0] == np.float32(np.float32(1e-12) / np.float32(448.0))
    assert (codes == 0).all()
    # above the floor the largest element of a row always maps to +-448 (code 0x7E / 0xFE)
    g = torch.Generator().manual_seed(12)
    x = (torch.randn(64, 256, generator=g) * torch.logspace(-9, 20, 64).unsqueeze(1)).numpy().astype(np.float32)
    codes, scales = oracle.quantize_rows_e4m3(x)
    idx = np.abs(x).argmax(axis=1)
    top = codes[np.arange(64), idx]
    assert ((top & 0x7F) == 0x7E).all()
    assert not ((codes & 0x7F) == 0x7F).any()           # never a NaN code


def test_quantiser_matches_the_generator_recipe_in_torch(oracle):
    """Same rows through torch's fp32 ops and CPU cast (the recipe that makes the synthetic caches)."""
    g = torch.Generator().manual_seed(13)
    x = torch.randn(500, 256, generator=g) * (torch.rand(500, 1, generator=g) * 20 + 1e-3)
    x[3] = 0.0
    c_ref, s_ref = W.quantize_e4m3_per_token(x)
    codes, scales = oracle.quantize_rows_e4m3(x.numpy())
    assert np.array_equal(scales, s_ref.numpy())
    assert np.array_equal(codes, c_ref.view(torch.uint8).numpy())


def test_dequantised_value_is_within_half_a_step(oracle):
    g = torch.Generator().manual_seed(14)
    x = (torch.randn(200, 256, generator=g) * 3).numpy().astype(np.float32)
    codes, scales = oracle.quantize_rows_e4m3(x)
    dec = np.vectorize(oracle.decode_e4m3fn)(codes)
    mag = np.abs(dec)
    step = np.where(mag < 2.0 ** -6, 2.0 ** -9, 2.0 ** (np.floor(np.log2(np.maximum(mag, 2.0 ** -6))) - 3))
    # the quotient itself is rounded once in fp32 before it is encoded: one more ulp of slack
    err = np.abs(dec - x.astype(np.float64) / scales.astype(np.float64)[:, None])
    assert (err <= 0.5 * step * (1 + 1e-6) + 1e-6).all()


def test_round_bf16_matches_torch(oracle):
    g = torch.Generator().manual_seed(15)
    x = torch.cat([torch.randn(5000, generator=g) * 1e3, torch.randn(5000, generator=g) * 1e-3,
                   torch.tensor([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40])])
    want = x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.round_bf16(x.numpy()), want)


@pytest.mark.parametrize("B,K,N", [(3, 40, 7), (5, 96, 130)])
def test_linear_matches_torch_fp64(oracle, B, K, N):
    g = torch.Generator().manual_seed(16 + B)
    a = torch.randn(B, K, generator=g).to(torch.bfloat16)
    w = (torch.randn(K, N, generator=g) * 0.1).to(torch.bfloat16)
    y = oracle.linear(oracle.bits_of(a), oracle.bits_of(w))
    ref = (a.double() @ w.double()).numpy()
    assert np.abs(y - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())
    # fp32 activations are taken as they are
    a32 = torch.randn(B, K, generator=g)
    y32 = oracle.linear(a32.numpy(), oracle.bits_of(w))
    assert np.abs(y32 - (a32.double() @ w.double()).numpy()).max() <= 1e-12 * max(1.0, np.abs(ref).max())


def test_linear_selects_weight_rows(oracle):
    """One-hot activations return rows of W exactly: pins the [in, out] layout and the operand order."""
    g = torch.Generator().manual_seed(17)
    w = torch.randn(12, 9, generator=g).to(torch.bfloat16)
    a = torch.zeros(4, 12, dtype=torch.bfloat16)
    for b, k in enumerate([0, 5, 11, 7]):
        a[b, k] = 2.0
    y = oracle.linear(oracle.bits_of(a), oracle.bits_of(w))
    for b, k in enumerate([0, 5, 11, 7]):
        assert np.array_equal(y[b], 2.0 * w[k].double().numpy())
