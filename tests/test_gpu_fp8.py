"""GPU parity for the fp8 (OCP e4m3, per-token fp32 scales) cache.  Parity is defined on the
dequantised values: oracle and GPU read the same codes and scales.  Tolerance: row-normalised max
error <= 3e-2 (fp32 accumulation, weights times value scale rounded to bf16)."""
import numpy as np
import pytest
import torch

import paper_2507_19427_amd as mfa
from paper_2507_19427_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("lens", [[1], [33], [64], [65], [1, 2, 64, 65, 700, 1500, 1023, 1024, 1025], [0, 5, 0, 300]])
def test_fp8_ragged_contiguous_with_poisoned_padding(lens):
    print(f"\n[case] fp8 ragged contiguous lens={lens}", flush=True)
    S = max(max(lens), 1) + 9
    case = W.make_contiguous_case("fp8", 200 + len(lens), B=len(lens), S=S, seq_lens=lens, kv_dtype="fp8", poison=True)
    ctx = U.get_ctx()
    got = U.run_gpu(ctx, case)
    ref = U.run_oracle(case)
    err = U.row_normalised_error(got, ref)
    print(f"   row-normalised max error {err:.3e}", flush=True)
    assert err <= U.TOL_FP8
    for b, L in enumerate(lens):
        if L == 0:
            assert (got[b] == 0).all()


def test_fp8_scales_matter():
    """Scaling one token's key scale must move the result the way the oracle says (scales are per token)."""
    print("\n[case] fp8 per-token scales", flush=True)
    case = W.make_contiguous_case("fp8s", 211, B=2, S=200, kv_dtype="fp8", poison=False)
    case.k_scale[0, 17] *= 6.0
    case.v_scale[1, 3] *= 0.25
    ctx = U.get_ctx()
    got = U.run_gpu(ctx, case)
    assert U.row_normalised_error(got, U.run_oracle(case)) <= U.TOL_FP8


def test_fp8_paged_equals_contiguous_bitwise_and_matches_oracle():
    print("\n[case] fp8 paged vs contiguous", flush=True)
    lens = [1, 64, 65, 200, 0, 127, 1000, 513]
    case = W.make_paged_case("fp8paged", 221, lens, kv_dtype="fp8", spare_pages=9, poison=True)
    contig = W.paged_to_contiguous(case, S=1024, poison=True)
    ctx = U.get_ctx()
    got_p = U.run_gpu(ctx, case, hint=1000)
    got_c = U.run_gpu(ctx, contig, hint=1000)
    assert np.array_equal(got_p, got_c)
    assert U.row_normalised_error(got_p, U.run_oracle(case)) <= U.TOL_FP8


def test_fp8_without_scales_is_rejected():
    case = W.make_contiguous_case("fp8e", 231, B=1, S=64, kv_dtype="fp8", poison=False)
    ctx = U.get_ctx()
    with pytest.raises(mfa.MfaError) as e:
        mfa.mfa_decode_attn(ctx, case.q.cuda(), case.k.cuda(), case.v.cuda(), case.seq_lens.cuda(), 64)
    assert e.value.status == mfa.MFA_ERR_INVALID_ARG


def test_fp8_run_to_run_determinism_and_prepared_calls():
    """Same inputs, same bits; and the pre-marshalled call objects bench.py uses give the same result as the
    checked wrappers (single query token and a pair)."""
    print("\n[case] fp8 determinism / prepared calls", flush=True)
    import paper_2507_19427_amd as mfa
    lens = [700, 64, 1500, 2, 129, 0]
    case = W.make_contiguous_case("fp8det", 911, B=len(lens), S=1504, seq_lens=lens, kv_dtype="fp8", poison=True)
    ctx = U.get_ctx()
    a = U.run_gpu(ctx, case)
    b = U.run_gpu(ctx, case)
    assert np.array_equal(a, b)
    d = U.to_dev
    q, k, v, ks, vs, sl = d(case.q), d(case.k), d(case.v), d(case.k_scale), d(case.v_scale), d(case.seq_lens)
    out = torch.empty(len(lens), 64, 256, dtype=torch.float32, device="cuda")
    call = mfa.PreparedDecodeAttn(ctx, q, k, v, sl, 1500, out, k_scale=ks, v_scale=vs)
    out.fill_(float("nan"))
    call()
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), a)
    qm = d(W.make_multi_query(case, 2, 912))
    want = mfa.mfa_decode_attn_multi(ctx, qm, k, v, sl, 1500, k_scale=ks, v_scale=vs)
    out2 = torch.full((len(lens), 2, 64, 256), float("nan"), dtype=torch.float32, device="cuda")
    call2 = mfa.PreparedDecodeAttn(ctx, qm, k, v, sl, 1500, out2, k_scale=ks, v_scale=vs)
    out2.fill_(float("nan"))
    call2()
    torch.cuda.synchronize()
    assert torch.equal(out2, want)
