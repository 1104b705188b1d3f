"""GPU parity for the 4-bit cache (Section 5.2: cache kept in 4 bits, attention computed in 8): e2m1 codes two
per byte with one fp32 scale per token and tensor.  The oracle dequantises the same bytes in fp64; tolerance as
for the 8-bit cache, since everything after the codes (two-term e4m3 query, bf16 weights) is the same."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2507_19427_amd as mfa
from paper_2507_19427_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _announce(name):
    print(f"\n[case] {name}", flush=True)


def _check(case, ctx, hint=None):
    got = U.run_gpu(ctx, case, hint=hint)
    err = U.row_normalised_error(got, U.run_oracle(case))
    print(f"   row-normalised max error {err:.3e}", flush=True)
    assert err <= U.TOL_FP8
    for b, L in enumerate(case.seq_lens.tolist()):
        if L == 0:
            assert (got[b] == 0).all()
    return got


@pytest.mark.parametrize("lens", [
    [5, 0, 1, 64, 65, 129, 128, 63],
    [0, 3000, 1, 0, 64, 2500, 129, 0, 2048, 65],
])
def test_fp4_mixed_lengths(lens):
    _announce(f"fp4 mixed lens={lens}")
    case = W.make_contiguous_case("fp4mixed", 800 + len(lens), B=len(lens), S=max(lens) + 8, seq_lens=lens, kv_dtype="fp4",
                                  poison=True)
    _check(case, U.get_ctx())


def test_fp4_more_sequences_than_workgroups():
    _announce("fp4 B=280 short ragged")
    g = torch.Generator().manual_seed(811)
    lens = torch.randint(1, 301, (280,), generator=g).tolist()
    for i in torch.randperm(280, generator=g)[:9].tolist():
        lens[i] = 0
    case = W.make_contiguous_case("fp4many", 812, B=280, S=304, seq_lens=lens, kv_dtype="fp4", poison=True)
    _check(case, U.get_ctx(max_batch=512, max_seq_len=4096))


def test_fp4_paged_bitwise_equal_to_contiguous():
    _announce("fp4 paged vs contiguous")
    g = torch.Generator().manual_seed(821)
    lens = torch.randint(1, 701, (70,), generator=g).tolist()
    lens[3], lens[11] = 0, 1
    case = W.make_paged_case("fp4paged", 822, lens, kv_dtype="fp4", spare_pages=9, poison=True)
    contig = W.paged_to_contiguous(case, S=704, poison=True)
    ctx = U.get_ctx()
    got_p = _check(case, ctx, hint=700)
    got_c = U.run_gpu(ctx, contig, hint=700)
    assert np.array_equal(got_p, got_c)


def test_fp4_key_and_value_bytes_are_taken_in_the_documented_order():
    """A sequence of one token: the output of every head is that token's value row, element by element (pins
    the nibble order and the chunk placement of V independently of K).  The weight 1 carries the value scale
    rounded to bf16, hence the 2^-8 relative allowance."""
    _announce("fp4 element order")
    B, S = 2, 64
    case = W.make_contiguous_case("fp4order", 831, B=B, S=S, seq_lens=[1, 64], kv_dtype="fp4", poison=False)
    got = U.run_gpu(U.get_ctx(), case)
    codes = torch.stack([case.v[0, 0] & 15, case.v[0, 0] >> 4], dim=-1).reshape(-1).long()
    table = torch.tensor([0, .5, 1, 1.5, 2, 3, 4, 6, -0.0, -.5, -1, -1.5, -2, -3, -4, -6], dtype=torch.float64)
    want = (table[codes] * float(case.v_scale[0, 0])).numpy()
    for h in range(64):
        assert np.allclose(got[0, h], want, rtol=2.0 ** -8, atol=0)


def test_fp4_two_query_tokens():
    _announce("fp4, two query tokens")
    lens = [0, 1500, 1, 2, 64, 129, 65, 700]
    case = W.make_contiguous_case("fp4mtp", 841, B=len(lens), S=1504, seq_lens=lens, kv_dtype="fp4", poison=True)
    qm = W.make_multi_query(case, 2, 842)
    d = U.to_dev
    out = mfa.mfa_decode_attn_multi(U.get_ctx(), d(qm), d(case.k), d(case.v), d(case.seq_lens), max(lens),
                                    d(case.k_scale), d(case.v_scale))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ref = np.stack([U.run_oracle(dataclasses.replace(case, q=qm[:, j].contiguous(),
                                                     seq_lens=torch.clamp(case.seq_lens - (1 - j), min=0).to(torch.int32)))
                    for j in range(2)], axis=1)
    err = U.row_normalised_error(got, ref)
    print(f"   row-normalised max error {err:.3e}", flush=True)
    assert err <= U.TOL_FP8


def test_fp4_at_full_size_on_sampled_rows():
    """B = 128, context 8192: the shape of the 8-bit benchmark configuration, in the launch bench.py times."""
    _announce("fp4 B=128 ctx=8192")
    case = W.make_contiguous_case("fp4big", 851, B=128, S=8192, kv_dtype="fp4", poison=False)
    got = U.run_gpu(U.get_ctx(), case)
    rows = U.sample_rows(case, 24, seed=6)
    ref = U.run_oracle(case, rows=rows)
    sel = np.stack([got[b, h] for b, h in rows])
    err = U.row_normalised_error(sel, ref)
    print(f"   row-normalised max error on {len(rows)} sampled rows {err:.3e}", flush=True)
    assert err <= U.TOL_FP8


def test_fp4_record_is_bit_exact_on_given_rows():
    """Quantisation decides integer codes: defined in single precision on both sides and compared bit for bit
    (contiguous and paged), including a zero row, signed zeros, exact midpoints and rows below the floor."""
    _announce("fp4 record, bit-exact")
    ctx = U.get_ctx()
    B, S = 96, 12
    g = torch.Generator().manual_seed(861)
    kv = torch.randn(B, 512, generator=g) * torch.logspace(-6, 6, B).unsqueeze(1)
    kv[5] = 0.0
    kv[6, ::2] = -0.0
    kv[7, :16] = torch.tensor([6.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, -0.25, -0.75, -1.25, -1.75, -2.5, -3.5, -5.0, -6.0])
    kv[7, 16:256] *= 0.1                                  # the key row's largest magnitude is 6: scale 1, exact ties
    kv[8] = 1e-20
    lens = torch.randint(0, S, (B,), generator=g, dtype=torch.int32)
    k = torch.full((B, S, 128), 0xEE, dtype=torch.uint8, device="cuda")
    v = k.clone()
    ks = torch.full((B, S), -1.0, dtype=torch.float32, device="cuda")
    vs = ks.clone()
    mfa.mfa_debug_kv_record(ctx, kv.cuda(), k, v, lens.cuda(), k_scale=ks, v_scale=vs)
    torch.cuda.synchronize()
    from oracle import mfa_oracle as O
    kc, ksc = O.quantize_rows_e2m1(kv[:, :256].numpy())
    vc, vsc = O.quantize_rows_e2m1(kv[:, 256:].numpy())
    kh, vh, ksh, vsh = k.cpu().numpy(), v.cpu().numpy(), ks.cpu().numpy(), vs.cpu().numpy()
    for b in range(B):
        L = int(lens[b])
        assert np.array_equal(kh[b, L], kc[b]) and np.array_equal(vh[b, L], vc[b]), b
        assert ksh[b, L] == ksc[b] and vsh[b, L] == vsc[b], b
        other = np.ones(S, dtype=bool)
        other[L] = False
        assert (kh[b, other] == 0xEE).all() and (vh[b, other] == 0xEE).all() and (ksh[b, other] == -1.0).all()
    # paged: same rows through a block table
    n_pages = B + 3
    table = torch.randperm(n_pages, generator=g)[:B].to(torch.int32).unsqueeze(1)
    kp = torch.full((n_pages, 64, 128), 0xEE, dtype=torch.uint8, device="cuda")
    vp = kp.clone()
    ksp = torch.full((n_pages, 64), -1.0, dtype=torch.float32, device="cuda")
    vsp = ksp.clone()
    mfa.mfa_debug_kv_record(ctx, kv.cuda(), kp, vp, lens.cuda(), k_scale=ksp, v_scale=vsp, block_table=table.cuda())
    torch.cuda.synchronize()
    kph, ksph = kp.cpu().numpy(), ksp.cpu().numpy()
    for b in range(B):
        assert np.array_equal(kph[int(table[b, 0]), int(lens[b])], kc[b]) and ksph[int(table[b, 0]), int(lens[b])] == ksc[b]


def test_fp4_append_then_attend():
    """Projection + 4-bit record + attention over the lengthened cache, against the oracle's chain with the
    record taken from the GPU's own fp32 projection tolerance: the dequantised record must lie within half a
    code step of the fp64 projection, and attention over the GPU-written cache must match the oracle over it."""
    _announce("fp4 append + attention")
    ctx = U.get_ctx()
    lens = [40, 0, 63, 64, 200]
    B, S = len(lens), 256
    case = W.make_contiguous_case("fp4app", 871, B=B, S=S, seq_lens=lens, kv_dtype="fp4", poison=False)
    g = torch.Generator().manual_seed(872)
    x = torch.randn(B, 7168, generator=g).to(torch.bfloat16)
    w_kv = (torch.randn(7168, 512, generator=g) * 0.02).to(torch.bfloat16)
    d = U.to_dev
    k, v, ks, vs = d(case.k), d(case.v), d(case.k_scale), d(case.v_scale)
    mfa.mfa_kv_append(ctx, d(x), d(w_kv), k, v, d(case.seq_lens), k_scale=ks, v_scale=vs)
    torch.cuda.synchronize()
    from oracle import mfa_oracle as O
    proj = O.linear(O.bits_of(x), O.bits_of(w_kv))                      # fp64 [B, 512]
    new = dataclasses.replace(case, k=k.cpu(), v=v.cpu(), k_scale=ks.cpu(), v_scale=vs.cpu(),
                              seq_lens=(case.seq_lens + 1).to(torch.int32))
    for b, L in enumerate(lens):
        for t, sc, off in ((new.k, new.k_scale, 0), (new.v, new.v_scale, 256)):
            packed = t[b, L].numpy()
            codes = np.stack([packed & 15, packed >> 4], axis=1).reshape(-1)
            dec = np.vectorize(O.decode_e2m1)(codes)
            mag = np.abs(dec)
            step = np.where(mag < 2.0, 0.5, np.where(mag < 4.0, 1.0, 2.0)) * float(sc[b, L])
            assert (np.abs(dec * float(sc[b, L]) - proj[b, off:off + 256]) <= 0.5 * step + 1e-3 * np.abs(proj[b]).max()).all()
        # rows before the new one are untouched
        assert torch.equal(new.k[b, :L], case.k[b, :L]) and torch.equal(new.v_scale[b, :L], case.v_scale[b, :L])
    got = U.run_gpu(ctx, new)
    err = U.row_normalised_error(got, U.run_oracle(new))
    print(f"   attention over the appended cache: row-normalised max error {err:.3e}", flush=True)
    assert err <= U.TOL_FP8
