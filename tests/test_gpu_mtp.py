"""GPU parity for a decode step with two query tokens per sequence (Section 5.2: multi-token prediction
multiplies the attention's arithmetic intensity, because the new tokens share one pass over the cache).
Query token j of q_len attends to the first L - (q_len - 1 - j) cached tokens, so the expected result is the
single-token oracle called once per query token with that length; nothing new is needed on the oracle's
side.  Same tolerances as the single-token tests."""
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


def _run_gpu(ctx, case, qm, hint=None):
    hint = int(hint if hint is not None else max(int(case.seq_lens.max()), 1))
    d = U.to_dev
    if case.paged:
        out = mfa.mfa_decode_attn_paged_multi(ctx, d(qm), d(case.k_pool), d(case.v_pool), d(case.block_table),
                                              d(case.seq_lens), hint, d(case.k_scale_pool), d(case.v_scale_pool))
    else:
        out = mfa.mfa_decode_attn_multi(ctx, d(qm), d(case.k), d(case.v), d(case.seq_lens), hint, d(case.k_scale),
                                        d(case.v_scale))
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _oracle(case, qm, rows=None):
    """[B, q_len, H, D] (or one row per sampled (b, h) and query token) from the single-token oracle."""
    q_len = qm.shape[1]
    outs = []
    for j in range(q_len):
        lens = torch.clamp(case.seq_lens - (q_len - 1 - j), min=0).to(torch.int32)
        outs.append(U.run_oracle(dataclasses.replace(case, q=qm[:, j].contiguous(), seq_lens=lens), rows=rows))
    return np.stack(outs, axis=1)


def _check(case, ctx, tol, hint=None, q_seed=900, q_len=2):
    qm = W.make_multi_query(case, q_len, q_seed)
    got = _run_gpu(ctx, case, qm, hint=hint)
    ref = _oracle(case, qm)
    err = U.row_normalised_error(got, ref)
    print(f"   row-normalised max error {err:.3e}", flush=True)
    assert err <= tol
    for b, L in enumerate(case.seq_lens.tolist()):
        if L == 0:
            assert (got[b] == 0).all()
        for j in range(q_len):
            if L < q_len - j:
                assert (got[b, j] == 0).all()      # this new token has nothing to attend to
    return got, qm


@pytest.mark.parametrize("lens", [
    [5, 0, 1, 2, 64, 65, 129, 128],
    [0, 3000, 1, 2, 64, 5000, 129, 65, 2048],
    [4096, 0, 0, 1, 0, 0, 0, 2],
    [63, 1, 1, 2, 1, 1, 2, 1, 1, 1, 2, 1, 1, 1, 1, 1, 1, 65],
])
def test_two_tokens_bf16_mixed_lengths(lens):
    _announce(f"two query tokens, bf16, lens={lens}")
    case = W.make_contiguous_case("mtp", 700 + len(lens), B=len(lens), S=max(lens) + 3, seq_lens=lens, poison=True)
    _check(case, U.get_ctx(), U.TOL_BF16)


def test_two_tokens_more_sequences_than_workgroups():
    _announce("two query tokens, B=300 short ragged")
    g = torch.Generator().manual_seed(711)
    lens = torch.randint(1, 201, (300,), generator=g).tolist()
    for i in torch.randperm(300, generator=g)[:15].tolist():
        lens[i] = 0
    case = W.make_contiguous_case("mtpmany", 712, B=300, S=208, seq_lens=lens, poison=True)
    _check(case, U.get_ctx(max_batch=512, max_seq_len=4096), U.TOL_BF16)


def test_two_tokens_fp8_mixed_lengths():
    _announce("two query tokens, fp8 mixed")
    lens = [0, 3000, 1, 2, 64, 2500, 129, 0, 2048, 65]
    case = W.make_contiguous_case("mtpfp8", 721, B=len(lens), S=3008, seq_lens=lens, kv_dtype="fp8", poison=True)
    _check(case, U.get_ctx(), U.TOL_FP8)


@pytest.mark.parametrize("kv_dtype,tol", [("bf16", U.TOL_BF16), ("fp8", U.TOL_FP8)])
def test_two_tokens_paged_bitwise_equal_to_contiguous(kv_dtype, tol):
    _announce(f"two query tokens, paged {kv_dtype} vs contiguous")
    g = torch.Generator().manual_seed(731)
    lens = torch.randint(1, 701, (70,), generator=g).tolist()
    lens[3], lens[11], lens[40] = 0, 1, 2
    case = W.make_paged_case("mtppaged", 732, lens, kv_dtype=kv_dtype, spare_pages=9, poison=True)
    contig = W.paged_to_contiguous(case, S=704, poison=True)
    ctx = U.get_ctx()
    got_p, qm = _check(case, ctx, tol, hint=700)
    got_c = _run_gpu(ctx, contig, qm, hint=700)
    assert np.array_equal(got_p, got_c)


def test_each_token_agrees_with_the_single_token_entry_point():
    """Token j of the two-token step against the one-token step run on the same query and its own length.
    The two launches visit the tokens in different groupings, so the bf16-rounded weights are taken against
    different running maxima: agreement to a fraction of the bf16 tolerance, not bitwise."""
    _announce("two-token step vs two one-token steps")
    lens = [777, 64, 1500, 2, 129]
    case = W.make_contiguous_case("mtpvs1", 741, B=len(lens), S=1504, seq_lens=lens, poison=True)
    ctx = U.get_ctx()
    qm = W.make_multi_query(case, 2, 742)
    got = _run_gpu(ctx, case, qm)
    for j in range(2):
        single = dataclasses.replace(case, q=qm[:, j].contiguous(), seq_lens=(case.seq_lens - (1 - j)).to(torch.int32))
        one = U.run_gpu(ctx, single, hint=max(lens))
        err = U.row_normalised_error(got[:, j], one.astype(np.float64))
        print(f"   token {j}: row-normalised max difference {err:.3e}", flush=True)
        assert err <= 0.5 * U.TOL_BF16


def test_one_token_through_the_multi_entry_point_is_the_single_token_path():
    _announce("q_len=1 through the multi entry point")
    lens = [300, 0, 65, 4000]
    case = W.make_contiguous_case("mtpq1", 751, B=4, S=4000, seq_lens=lens, poison=True)
    ctx = U.get_ctx()
    a = U.run_gpu(ctx, case)
    b = _run_gpu(ctx, case, case.q.unsqueeze(1).contiguous())
    assert np.array_equal(a, b[:, 0])


@pytest.mark.parametrize("q_len", [3, 4])
@pytest.mark.parametrize("kv_dtype,tol", [("bf16", U.TOL_BF16), ("fp8", U.TOL_FP8)])
def test_three_and_four_tokens(q_len, kv_dtype, tol):
    """Three and four query tokens: one pass over a bf16 cache (the kernel that keeps all query tokens of a sequence
    in one wave); pair by pair over the 8-bit cache, an odd count ending with an overlapping pair."""
    _announce(f"{q_len} query tokens, {kv_dtype}")
    lens = [0, 1, 2, 3, 4, 64, 65, 66, 67, 129, 1500, 700]
    case = W.make_contiguous_case("mtp34", 780 + q_len, B=len(lens), S=1504, seq_lens=lens, kv_dtype=kv_dtype, poison=True)
    _check(case, U.get_ctx(), tol, q_len=q_len)


def test_four_tokens_paged_bitwise_equal_to_contiguous():
    _announce("4 query tokens, paged vs contiguous")
    g = torch.Generator().manual_seed(791)
    lens = torch.randint(1, 401, (40,), generator=g).tolist()
    lens[2], lens[7], lens[9] = 0, 2, 3
    case = W.make_paged_case("mtp4paged", 792, lens, spare_pages=5, poison=True)
    contig = W.paged_to_contiguous(case, S=448, poison=True)
    ctx = U.get_ctx()
    got_p, qm = _check(case, ctx, U.TOL_BF16, hint=400, q_len=4)
    assert np.array_equal(got_p, _run_gpu(ctx, contig, qm, hint=400))


@pytest.mark.parametrize("q_len", [3, 4])
def test_one_pass_kernel_restarts_a_segment_whose_scores_outrun_the_reference(q_len):
    """The one-pass kernel fixes a head's reference exponent at its first unit and starts the segment again with
    a higher one when a later score exceeds it by more than 2^40.  Planted: keys aligned with the queries of some
    heads, far into the sequence and in different tiles, whose scores lie 60 to 140 (natural units) above the
    rest -- for a few heads of one head group only, for all heads, twice in a row (a second, larger outlier after
    the first), and in the last tile.  The result must be the usual softmax: practically the outlier's value row."""
    _announce(f"{q_len} query tokens, outlier scores force restarts")
    lens = [700, 300, 130, 2000]
    case = W.make_contiguous_case("mtprestart", 795 + q_len, B=len(lens), S=2000, seq_lens=lens, poison=True)
    qm = W.make_multi_query(case, q_len, 796)
    k = case.k.float()
    qf = qm.float()

    def plant(b, pos, heads, tok, gain):
        # key row pos of sequence b := gain * (mean of the chosen heads' queries of query token tok), so that
        # those heads score about gain * |q|^2 / 16 on it
        qv = qf[b, tok, heads].mean(0)
        k[b, pos] = gain * qv / qv.norm() ** 2 * 16.0 * len(heads) ** 0.0

    plant(0, 333, [3, 4, 5], 0, 60.0)                    # one head group only: the other waves must restart with it
    plant(1, 77, list(range(64)), q_len - 1, 30.0)       # weak for most heads (mean over 64 queries): may or may not trip
    plant(2, 70, [17], 1, 80.0)
    plant(2, 127, [17], 1, 140.0)                        # a second, larger outlier later in the same sequence
    plant(3, 1990, [60, 61, 62, 63], 0, 100.0)           # in the last tile of a long sequence cut over workgroups
    case.k = k.to(torch.bfloat16)
    got = _run_gpu(U.get_ctx(), case, qm)
    ref = _oracle(case, qm)
    err = U.row_normalised_error(got, ref)
    print(f"   row-normalised max error {err:.3e}", flush=True)
    assert err <= U.TOL_BF16
    # the planted key dominates its head: the output is that token's value row
    assert np.abs(got[0, 0, 4] - case.v[0, 333].float().numpy()).max() <= 1e-2 * np.abs(case.v[0, 333].float().numpy()).max()
    assert np.array_equal(got, _run_gpu(U.get_ctx(), case, qm))           # and bitwise reproducible


@pytest.mark.parametrize("q_len", [3, 4])
def test_three_and_four_tokens_at_benchmark_size_on_sampled_rows(q_len):
    """B = 64, context 4096 (the benchmark's cache), one pass for three and for four query tokens."""
    _announce(f"{q_len} query tokens at B=64 ctx=4096")
    ctx = U.get_ctx()
    case = W.config2_step3(poison=False)
    qm = W.make_multi_query(case, q_len, 797)
    got = _run_gpu(ctx, case, qm)
    assert np.isfinite(got).all()
    rows = U.sample_rows(case, 24)
    ref = _oracle(case, qm, rows=rows)                                  # [rows, q_len, D] stacked on axis 1
    sub = np.stack([got[b, :, h] for b, h in rows])
    err = U.row_normalised_error(sub, ref)
    print(f"   sampled rows {len(rows)} x {q_len} tokens: row-normalised max error {err:.3e}", flush=True)
    assert err <= U.TOL_BF16


def test_four_tokens_beyond_the_one_pass_kernels_batch_limit_fall_back_to_pairs():
    _announce("4 query tokens, B=600 (pairs)")
    g = torch.Generator().manual_seed(798)
    lens = torch.randint(0, 90, (600,), generator=g).tolist()
    case = W.make_contiguous_case("mtp600", 799, B=600, S=96, seq_lens=lens, poison=True)
    _check(case, U.get_ctx(max_batch=1024, max_seq_len=4096), U.TOL_BF16, q_len=4)


def test_unsupported_query_counts_are_refused():
    _announce("q_len=5 and q_len=2 on fixed splits are refused")
    case = W.make_contiguous_case("mtpbad", 761, B=2, S=64, seq_lens=[64, 10], poison=True)
    q3 = W.make_multi_query(case, 5, 762)
    with pytest.raises(mfa.MfaError) as ei:
        _run_gpu(U.get_ctx(), case, q3)
    assert ei.value.status == mfa.MFA_ERR_UNSUPPORTED
    ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=16, max_seq_len=8192, schedule=mfa.MFA_SCHEDULE_FIXED))
    with pytest.raises(mfa.MfaError) as ei:
        _run_gpu(ctx, case, W.make_multi_query(case, 2, 763))
    assert ei.value.status == mfa.MFA_ERR_UNSUPPORTED
    ctx.close()


def test_two_tokens_at_benchmark_size_on_sampled_rows():
    """B = 64, context 4096 (the benchmark's shape and launch configuration), bf16 and fp8."""
    _announce("two query tokens at B=64 ctx=4096")
    ctx = U.get_ctx()
    for kv_dtype, tol in (("bf16", U.TOL_BF16), ("fp8", U.TOL_FP8)):
        case = W.make_contiguous_case("mtpbig", 771, B=64, S=4096, kv_dtype=kv_dtype, poison=False)
        qm = W.make_multi_query(case, 2, 772)
        got = _run_gpu(ctx, case, qm)
        rows = U.sample_rows(case, 24, seed=5)
        ref = _oracle(case, qm, rows=rows)                              # [n_rows, 2, D]
        sel = np.stack([got[b, :, h] for b, h in rows])
        err = U.row_normalised_error(sel, ref)
        print(f"   {kv_dtype}: row-normalised max error on {len(rows)} sampled rows {err:.3e}", flush=True)
        assert err <= tol
