"""Pins for the oracle's own bf16 / e4m3fn decoders and bf16 encoder: exhaustive code tables
against torch's CPU casts (a library routine), plus hand-computed codes."""
import math
from fractions import Fraction

import numpy as np
import torch


def _same(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.array_equal(np.isnan(a), np.isnan(b)) and np.array_equal(a[~np.isnan(a)], b[~np.isnan(b)]) \
        and np.array_equal(np.signbit(a[~np.isnan(a)]), np.signbit(b[~np.isnan(b)]))


def test_bf16_decode_all_codes(oracle):
    ref = torch.arange(65536, dtype=torch.int32).to(torch.int16).view(torch.bfloat16).to(torch.float64).numpy()
    mine = [oracle.decode_bf16(i) for i in range(65536)]
    assert _same(mine, ref)


def test_e4m3fn_decode_all_codes(oracle):
    ref = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = [oracle.decode_e4m3fn(i) for i in range(256)]
    assert _same(mine, ref)


def test_e4m3fn_hand_codes(oracle):
    # values worked out from the format definition: bias 7, 3 fraction bits, no infinity
    assert oracle.decode_e4m3fn(0x00) == 0.0
    assert oracle.decode_e4m3fn(0x01) == 2.0 ** -9          # smallest subnormal
    assert oracle.decode_e4m3fn(0x07) == 7 * 2.0 ** -9      # largest subnormal
    assert oracle.decode_e4m3fn(0x08) == 2.0 ** -6          # smallest normal
    assert oracle.decode_e4m3fn(0x38) == 1.0
    assert oracle.decode_e4m3fn(0x7E) == 448.0              # largest finite
    assert oracle.decode_e4m3fn(0xFE) == -448.0
    assert math.isnan(oracle.decode_e4m3fn(0x7F)) and math.isnan(oracle.decode_e4m3fn(0xFF))
    assert oracle.decode_e4m3fn(0x78) == 256.0              # exponent 15 is finite except fraction 7


def test_bf16_hand_codes(oracle):
    assert oracle.decode_bf16(0x3F80) == 1.0
    assert oracle.decode_bf16(0xC000) == -2.0
    assert oracle.decode_bf16(0x0001) == 2.0 ** -133
    assert oracle.decode_bf16(0x7F7F) == (2 - 2.0 ** -7) * 2.0 ** 127
    assert math.isinf(oracle.decode_bf16(0x7F80)) and math.isnan(oracle.decode_bf16(0x7FC0))


def test_bf16_encode_is_nearest_even(oracle):
    """Exact check with rationals: the encoded value is a nearest bf16, and on ties the even code."""
    rng = np.random.default_rng(0)
    xs = list(rng.standard_normal(2000) * np.exp(rng.standard_normal(2000) * 10))
    # exact ties and near ties around 1.0 (spacing 2^-7): halfway points
    for k in range(16):
        xs += [1.0 + (2 * k + 1) * 2.0 ** -8, 1.0 + (2 * k + 1) * 2.0 ** -8 * (1 + 2.0 ** -40),
               -(1.0 + (2 * k + 1) * 2.0 ** -8)]
    xs += [0.0, -0.0, 2.0 ** -133, 2.0 ** -134, 3 * 2.0 ** -134, 2.0 ** -126 * (1 - 2.0 ** -9), 1e-45, 3.3e38, 3.4e38]
    for x in xs:
        code = oracle.encode_bf16(float(x))
        got = oracle.decode_bf16(code)
        if math.isinf(got):
            assert abs(x) >= (2 - 2.0 ** -8) * 2.0 ** 127
            continue
        lo = oracle.decode_bf16(code - 1) if (code & 0x7FFF) > 0 else None
        hi = oracle.decode_bf16(code + 1)
        err = abs(Fraction(got) - Fraction(float(x)))
        for nb in (lo, hi):
            if nb is None or math.isinf(nb) or math.isnan(nb):
                continue
            e2 = abs(Fraction(nb) - Fraction(float(x)))
            assert err <= e2
            if err == e2:
                assert code % 2 == 0, (x, hex(code))
        assert (code >> 15) == (1 if math.copysign(1.0, x) < 0 else 0)


def test_bf16_encode_matches_torch_on_floats(oracle):
    g = torch.Generator().manual_seed(3)
    xs = torch.randn(20000, generator=g) * torch.exp(torch.randn(20000, generator=g) * 8)
    ref = xs.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    mine = np.array([oracle.encode_bf16(float(v)) for v in xs.double().numpy()], dtype=np.uint16)
    assert np.array_equal(ref, mine)
