"""The attention entry point that allocates nothing (mfa_decode_attn_static: partial results in the library's
fixed device array) against mfa_decode_attn on the same inputs, through the C boundary: two calls in a row, the
second with a smaller input, so that whatever the first call left in the shared array must not leak into the
second.  Same kernels, same schedule: the two entry points must agree bit for bit, and both are held to the
oracle's tolerance."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2507_19427_amd as mfa
from paper_2507_19427_amd import workloads as W

from gpu_util import TOL_BF16, TOL_FP8, get_ctx, row_normalised_error, run_oracle, to_dev

pytestmark = pytest.mark.gpu


def _both(ctx, case, hint):
    q, k, v, lens = to_dev(case.q), to_dev(case.k), to_dev(case.v), to_dev(case.seq_lens)
    ks, vs = to_dev(case.k_scale), to_dev(case.v_scale)
    ref = mfa.mfa_decode_attn(ctx, q, k, v, lens, hint, ks, vs)
    out = torch.full_like(ref, float("nan"))
    mfa.mfa_decode_attn_static(ctx, q, k, v, lens, hint, out, ks, vs)
    torch.cuda.synchronize()
    return out.cpu().numpy(), ref.cpu().numpy()


@pytest.mark.parametrize("kv_dtype,tol", [("bf16", TOL_BF16), ("fp8", TOL_FP8)])
def test_static_scratch_entry_matches_workspace_entry_twice(kv_dtype, tol):
    ctx = get_ctx(max_batch=128, max_seq_len=8192)
    # first call: several sequences cut over many workgroups (every partial slot of the call is written)
    big = W.make_contiguous_case("noalloc_big", 21, B=6, S=2100, seq_lens=[2100, 1, 777, 0, 64, 1500],
                                 kv_dtype=kv_dtype, poison=True)
    got, ref = _both(ctx, big, 2100)
    assert np.array_equal(got, ref)
    assert row_normalised_error(got, run_oracle(big)) <= tol
    # second call, smaller: fewer sequences, fewer tiles, other slots in use
    small = W.make_contiguous_case("noalloc_small", 22, B=2, S=300, seq_lens=[300, 129], kv_dtype=kv_dtype, poison=True)
    got, ref = _both(ctx, small, 300)
    assert np.array_equal(got, ref)
    assert row_normalised_error(got, run_oracle(small)) <= tol


def test_static_scratch_entry_refuses_what_does_not_fit():
    ctx = get_ctx(max_batch=256, max_seq_len=1024)
    B = 129                                             # one more sequence than the fixed array is sized for
    q = torch.zeros(B, 64, 256, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(B, 64, 256, dtype=torch.bfloat16, device="cuda")
    lens = torch.full((B,), 64, dtype=torch.int32, device="cuda")
    out = torch.zeros(B, 64, 256, dtype=torch.float32, device="cuda")
    with pytest.raises(mfa.MfaError) as e:
        mfa.mfa_decode_attn_static(ctx, q, k, k, lens, 64, out)
    assert e.value.status == mfa.MFA_ERR_WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0               # nothing was launched
