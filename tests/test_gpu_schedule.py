"""GPU parity for the way work is spread over workgroups.  The balanced schedule lays the tiles of all
sequences end to end and gives every workgroup an equal range, so a workgroup may hold the end of one
sequence, several whole sequences and the start of another; sequences without tokens belong to nobody.
These cases exercise those boundaries, the fixed-split schedule that remains for very large batches,
and the agreement of the two.  Same oracle, same tolerances as the other parity tests."""
import numpy as np
import pytest
import torch

import paper_2507_19427_amd as mfa
from paper_2507_19427_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _announce(name):
    print(f"\n[case] {name}", flush=True)


def _lens(seed, B, lo, hi, zeros=0):
    g = torch.Generator().manual_seed(seed)
    lens = torch.randint(lo, hi + 1, (B,), generator=g).tolist()
    for i in torch.randperm(B, generator=g)[:zeros].tolist():
        lens[i] = 0
    return lens


def _check(case, ctx, tol, hint=None):
    got = U.run_gpu(ctx, case, hint=hint)
    err = U.row_normalised_error(got, U.run_oracle(case))
    print(f"   row-normalised max error {err:.3e}", flush=True)
    assert err <= tol
    for b, L in enumerate(case.seq_lens.tolist()):
        if L == 0:
            assert (got[b] == 0).all()
    return got


def test_more_sequences_than_workgroups():
    """300 short sequences on 256 workgroups: most workgroups hold pieces of two or three sequences."""
    _announce("B=300 short ragged, some empty")
    lens = _lens(301, 300, 1, 200, zeros=17)
    case = W.make_contiguous_case("many", 302, B=300, S=208, seq_lens=lens, poison=True)
    ctx = U.get_ctx(max_batch=512, max_seq_len=4096)
    _check(case, ctx, U.TOL_BF16)


@pytest.mark.parametrize("lens", [
    [0, 3000, 1, 0, 64, 5000, 129, 0, 2048],
    [0, 0, 0, 1],
    [4096, 0, 0, 0, 0, 0, 0, 1],
    [63, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 65],
])
def test_mixed_lengths_cross_workgroup_boundaries(lens):
    _announce(f"mixed lens={lens}")
    S = max(lens) + 5
    case = W.make_contiguous_case("mixed", 310 + len(lens), B=len(lens), S=S, seq_lens=lens, poison=True)
    _check(case, U.get_ctx(), U.TOL_BF16)


def test_fewer_tiles_than_workgroups_and_hint_far_above_lengths():
    """The grid is sized from the hint; with short sequences most workgroups find an empty range."""
    _announce("tiny lens under a large hint")
    lens = [70, 1, 0, 130]
    case = W.make_contiguous_case("tinyhint", 321, B=4, S=256, seq_lens=lens, poison=True)
    _check(case, U.get_ctx(), U.TOL_BF16, hint=256)
    ctx = U.get_ctx(max_batch=128, max_seq_len=32768)
    q, lens_d = case.q.cuda(), case.seq_lens.cuda()
    k = torch.full((4, 30000, 256), float("nan"), dtype=torch.bfloat16)
    v = k.clone()
    k[:, :256], v[:, :256] = case.k, case.v
    out = mfa.mfa_decode_attn(ctx, q, k.cuda(), v.cuda(), lens_d, 30000)
    torch.cuda.synchronize()
    assert U.row_normalised_error(out.cpu().numpy(), U.run_oracle(case)) <= U.TOL_BF16


def test_paged_ragged_many_sequences_bitwise_equal_to_contiguous():
    _announce("paged B=160 ragged vs contiguous")
    lens = _lens(331, 160, 1, 700, zeros=5)
    case = W.make_paged_case("pagedmany", 332, lens, spare_pages=11, poison=True)
    contig = W.paged_to_contiguous(case, S=704, poison=True)
    ctx = U.get_ctx(max_batch=512, max_seq_len=4096)
    got_p = _check(case, ctx, U.TOL_BF16, hint=700)
    got_c = U.run_gpu(ctx, contig, hint=700)
    assert np.array_equal(got_p, got_c)


@pytest.mark.parametrize("lens", [
    [6000] + [3] * 63,                                   # one sequence holds nearly every tile: its pieces span all dies
    [1] * 56 + [2500] * 8,                               # all the work in the last eighth of the rows
    [700, 0, 0, 0, 0, 0, 0, 9000] * 2,                   # 16 rows, two long ones per eight
    [300 + 37 * i for i in range(64)],                   # steadily growing lengths
])
def test_merge_row_placement_is_only_a_matter_of_speed(lens):
    """The merge kernel hands its workgroups the rows that a batch of equal lengths would have left on their own die.
    With lengths as unequal as these the guess is wrong for most rows; the result must not depend on it.  Batches whose
    size is a multiple of 8 with at least 256 tiles, so that the placement is in force."""
    _announce(f"skewed lengths, B={len(lens)}")
    case = W.make_contiguous_case("skew", 360 + len(lens), B=len(lens), S=max(lens) + 2, seq_lens=lens, poison=True)
    got = _check(case, U.get_ctx(), U.TOL_BF16)
    assert np.array_equal(got, U.run_gpu(U.get_ctx(), case))
    fixed = U.get_ctx(schedule=mfa.MFA_SCHEDULE_FIXED)  # another schedule, another merge order: same rows within tolerance
    assert U.row_normalised_error(U.run_gpu(fixed, case), U.run_oracle(case)) <= U.TOL_BF16


def test_fp8_more_sequences_than_workgroups():
    _announce("fp8 B=280 short ragged")
    lens = _lens(341, 280, 1, 300, zeros=9)
    case = W.make_contiguous_case("fp8many", 342, B=280, S=304, seq_lens=lens, kv_dtype="fp8", poison=True)
    ctx = U.get_ctx(max_batch=512, max_seq_len=4096)
    _check(case, ctx, U.TOL_FP8)


def test_fp8_mixed_lengths():
    _announce("fp8 mixed")
    lens = [0, 3000, 1, 0, 64, 2500, 129, 0, 2048, 65]
    case = W.make_contiguous_case("fp8mixed", 343, B=len(lens), S=3008, seq_lens=lens, kv_dtype="fp8", poison=True)
    _check(case, U.get_ctx(), U.TOL_FP8)


@pytest.mark.parametrize("B,hi,kv_dtype", [(1000, 150, "bf16"), (4096, 70, "bf16"), (700, 200, "fp8")])
def test_batches_between_513_and_4096_sequences(B, hi, kv_dtype):
    """Above 512 sequences the lengths are scanned cooperatively through LDS instead of by every wave alone;
    4096 is the largest batch the balanced schedule takes."""
    _announce(f"B={B} {kv_dtype}, lengths 1..{hi}, some empty")
    lens = _lens(400 + B, B, 1, hi, zeros=B // 20)
    lens[0], lens[B - 1] = 0, hi                     # an empty first sequence, a full last one
    case = W.make_contiguous_case("large", 401 + B, B=B, S=hi + 2, seq_lens=lens, kv_dtype=kv_dtype, poison=True)
    ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=B, max_seq_len=256))
    _check(case, ctx, U.TOL_FP8 if kv_dtype == "fp8" else U.TOL_BF16)
    ctx.close()


def test_two_query_tokens_with_a_thousand_sequences():
    _announce("B=1000, two query tokens")
    B = 1000
    lens = _lens(451, B, 1, 130, zeros=40)
    case = W.make_contiguous_case("large2", 452, B=B, S=136, seq_lens=lens, poison=True)
    qm = W.make_multi_query(case, 2, 453)
    ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=B, max_seq_len=256))
    out = mfa.mfa_decode_attn_multi(ctx, qm.cuda(), case.k.cuda(), case.v.cuda(), case.seq_lens.cuda(), 130)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    import dataclasses
    ref = np.stack([U.run_oracle(dataclasses.replace(case, q=qm[:, j].contiguous(),
                                                     seq_lens=torch.clamp(case.seq_lens - (1 - j), min=0).to(torch.int32)))
                    for j in range(2)], axis=1)
    assert U.row_normalised_error(got, ref) <= U.TOL_BF16
    ctx.close()


def test_fixed_split_schedule_agrees(monkeypatch):
    """schedule = MFA_SCHEDULE_FIXED selects the schedule with equal chunks per sequence; both must match the
    oracle.  The environment override (MFA_SCHEDULE=fixed at context creation) selects the same code path."""
    _announce("fixed-split schedule")
    lens = [0, 3000, 1, 64, 5000, 129, 2048]
    case = W.make_contiguous_case("fixed", 351, B=len(lens), S=5008, seq_lens=lens, poison=True)
    ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=16, max_seq_len=8192, schedule=mfa.MFA_SCHEDULE_FIXED))
    got_fixed = _check(case, ctx, U.TOL_BF16)
    ctx.close()
    monkeypatch.setenv("MFA_SCHEDULE", "fixed")
    ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=16, max_seq_len=8192))
    got_env = _check(case, ctx, U.TOL_BF16)
    ctx.close()
    monkeypatch.delenv("MFA_SCHEDULE")
    assert np.array_equal(got_fixed, got_env)
    got_bal = _check(case, U.get_ctx(), U.TOL_BF16)
    assert U.row_normalised_error(got_fixed, got_bal.astype(np.float64)) <= U.TOL_BF16


def test_batch_above_the_balanced_limit_uses_fixed_splits():
    """Batches of more than 4096 sequences fall back to one workgroup per sequence."""
    _announce("B=4100")
    B = 4100
    lens = _lens(361, B, 1, 64, zeros=31)
    case = W.make_contiguous_case("huge", 362, B=B, S=64, seq_lens=lens, poison=True)
    ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=B, max_seq_len=64))
    _check(case, ctx, U.TOL_BF16)
    ctx.close()


def test_balanced_run_to_run_determinism():
    _announce("balanced determinism")
    lens = _lens(371, 200, 1, 900, zeros=3)
    case = W.make_contiguous_case("det2", 372, B=200, S=904, seq_lens=lens, poison=True)
    ctx = U.get_ctx(max_batch=512, max_seq_len=4096)
    a = U.run_gpu(ctx, case)
    b = U.run_gpu(ctx, case)
    assert np.array_equal(a, b)
