"""The named workloads at their full size, in the launch configuration the benchmark times:
sampled (sequence, head) rows against the oracle, plus properties that hold at any size."""
import numpy as np
import pytest
import torch

import paper_2507_19427_amd as mfa
from paper_2507_19427_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _check_sampled(case, got, n_rows, tol):
    rows = U.sample_rows(case, n_rows)
    ref = U.run_oracle(case, rows=rows)
    sub = np.stack([got[b, h] for b, h in rows])
    err = U.row_normalised_error(sub, ref)
    print(f"[{case.name}] sampled rows {len(rows)}: row-normalised max error {err:.3e}", flush=True)
    assert err <= tol


def _check_convex(case_v, lens, got):
    """Every output element lies between the min and max of its value column."""
    for b in (0, len(lens) - 1):
        L = int(lens[b])
        v = case_v(b, L)
        assert (got[b] <= v.max(0) + 1e-5).all() and (got[b] >= v.min(0) - 1e-5).all()


def test_config2_b64_ctx4096():
    print("\n[case] cfg2 B=64 ctx=4096 bf16 contiguous", flush=True)
    case = W.config2_step3(poison=False)
    ctx = U.get_ctx()
    assert mfa.mfa_decode_num_splits(ctx, 64, 4096) == 4
    got = U.run_gpu(ctx, case)
    assert np.isfinite(got).all()
    # every one of the 64 x 64 rows against the oracle (a few seconds on the machine's host cores)
    err = U.row_normalised_error(got, U.run_oracle(case))
    print(f"[{case.name}] all {64 * 64} rows: row-normalised max error {err:.3e}", flush=True)
    assert err <= U.TOL_BF16
    _check_convex(lambda b, L: case.v[b, :L].float().numpy(), case.seq_lens, got)
    again = U.run_gpu(ctx, case)
    assert np.array_equal(got, again)


def _exact_grid_case(name, seed, B, S):
    """Keys and values on a coarse grid (multiples of 1/8 up to 4 in magnitude), so that a key plus an integer
    shift is again a bf16 value: the shifted cache holds exactly K + delta."""
    case = W.make_contiguous_case(name, seed, B=B, S=S, poison=False)
    grid = lambda t: (torch.clamp(torch.round(t.float() * 8), -32, 32) / 8).to(torch.bfloat16)
    case.k, case.v = grid(case.k), grid(case.v)
    return case


@pytest.mark.parametrize("B,S", [(64, 4096), (16, 32768)])
def test_size_independent_properties_at_full_size(B, S):
    """Properties of softmax attention that hold at any size, on the benchmark's shape and the long-context one,
    in the launch configuration the benchmark times:
      Q = 0                        ->  the output is the mean of the cached values;
      a constant added to all keys ->  the output does not change (the softmax is shift invariant);
      tokens permuted (K and V alike) -> the output does not change."""
    print(f"\n[case] properties at B={B} ctx={S}", flush=True)
    ctx = U.get_ctx()
    case = _exact_grid_case("props", 71, B, S)
    q, k, v, lens = case.q.cuda(), case.k.cuda(), case.v.cuda(), case.seq_lens.cuda()
    run = lambda q_, k_, v_: mfa.mfa_decode_attn(ctx, q_, k_, v_, lens, S).cpu().numpy()
    base = run(q, k, v)
    assert np.isfinite(base).all()

    mean_v = v.float().mean(dim=1).cpu().numpy()                       # [B, 256]
    got0 = run(torch.zeros_like(q), k, v)
    err0 = U.row_normalised_error(got0, np.broadcast_to(mean_v[:, None, :], got0.shape))
    print(f"   Q = 0 against mean(V): {err0:.3e}", flush=True)
    assert err0 <= 1e-4                                                # equal weights are exact; fp32 summation order only

    delta = torch.zeros(256, dtype=torch.bfloat16, device="cuda")
    delta[::3] = 1.0
    delta[1::5] = -2.0
    k_shift = (k.float() + delta.float()).to(torch.bfloat16)
    assert torch.equal(k_shift.float(), k.float() + delta.float())     # the shifted keys are exact
    err_shift = U.row_normalised_error(run(q, k_shift, v), base)
    print(f"   keys shifted by a constant vector: {err_shift:.3e}", flush=True)
    assert err_shift <= U.TOL_BF16                                      # two results, each within the tolerance of the exact one

    perm = torch.randperm(S, generator=torch.Generator().manual_seed(72)).cuda()
    err_perm = U.row_normalised_error(run(q, k[:, perm].contiguous(), v[:, perm].contiguous()), base)
    print(f"   tokens permuted: {err_perm:.3e}", flush=True)
    assert err_perm <= U.TOL_BF16


def test_config3_ragged_paged():
    print("\n[case] cfg3 128 ragged paged sequences", flush=True)
    case = W.config3_ragged_paged(poison=True)
    assert case.B == 128 and int(case.seq_lens.min()) >= 1024 and int(case.seq_lens.max()) <= 8192
    ctx = U.get_ctx()
    got = U.run_gpu(ctx, case, hint=8192)
    assert np.isfinite(got).all()
    _check_sampled(case, got, 64, U.TOL_BF16)


def test_config4_b16_ctx32768():
    print("\n[case] cfg4 B=16 ctx=32768 bf16 contiguous", flush=True)
    case = W.config4_long(poison=False)
    ctx = U.get_ctx()
    assert mfa.mfa_decode_num_splits(ctx, 16, 32768) == 16
    got = U.run_gpu(ctx, case)
    assert np.isfinite(got).all()
    _check_sampled(case, got, 32, U.TOL_BF16)
    _check_convex(lambda b, L: case.v[b, :L].float().numpy(), case.seq_lens, got)


def test_two_very_long_sequences():
    """131,072 tokens per sequence (four times the longest named context): one sequence is cut over 128
    workgroups, 2048 tiles in all; sampled rows against the oracle, bf16 and fp8."""
    print("\n[case] B=2 ctx=131072", flush=True)
    ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=2, max_seq_len=131072))
    for kv_dtype, tol in (("bf16", U.TOL_BF16), ("fp8", U.TOL_FP8)):
        case = W.make_contiguous_case("verylong", 61, B=2, S=131072, seq_lens=[131072, 100001], kv_dtype=kv_dtype, poison=True)
        got = U.run_gpu(ctx, case, hint=131072)
        assert np.isfinite(got).all()
        rows = [(0, 0), (0, 63), (1, 17), (1, 40), (0, 31), (1, 5)]
        ref = U.run_oracle(case, rows=rows)
        sub = np.stack([got[b, h] for b, h in rows])
        err = U.row_normalised_error(sub, ref)
        print(f"   {kv_dtype}: row-normalised max error on {len(rows)} sampled rows {err:.3e}", flush=True)
        assert err <= tol
    ctx.close()
