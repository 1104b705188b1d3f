"""GPU parity: the HIP decode attention, called through the C boundary, against the CPU oracle on
the same seeded bytes.  Tolerance: row-normalised max error <= 1e-2 for a bf16 cache (fp32
accumulation, attention weights rounded to bf16 before the value product)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2507_19427_amd as mfa
from paper_2507_19427_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _announce(name):
    print(f"\n[case] {name}", flush=True)


def test_library_is_loaded_in_tree():
    import os
    p = mfa.binding.lib_path()
    assert os.path.exists(p) and os.path.dirname(p).endswith("paper_2507_19427_amd")
    assert mfa.binding.lib() is not None


def test_config1_tiny_full_compare():
    _announce("cfg1 tiny B=2 ctx=256")
    case = W.config1_tiny()
    ctx = U.get_ctx()
    got = U.run_gpu(ctx, case)
    ref = U.run_oracle(case)
    assert got.shape == (2, 64, 256) and got.dtype == np.float32
    assert U.row_normalised_error(got, ref) <= U.TOL_BF16


@pytest.mark.parametrize("lens", [
    [1], [31], [32], [33], [63], [64], [65], [127, 128, 129],
    [1, 2, 64, 65, 700, 1500, 1023, 1024, 1025],
    [0, 5, 0, 300],
])
def test_ragged_contiguous_with_poisoned_padding(lens):
    _announce(f"ragged contiguous lens={lens}")
    S = max(max(lens), 1) + 7            # padding rows past the longest sequence, all NaN
    case = W.make_contiguous_case("ragged", 100 + len(lens), B=len(lens), S=S, seq_lens=lens, poison=True)
    ctx = U.get_ctx()
    got = U.run_gpu(ctx, case)
    ref = U.run_oracle(case)
    assert U.row_normalised_error(got, ref) <= U.TOL_BF16
    for b, L in enumerate(lens):
        if L == 0:
            assert (got[b] == 0).all()
        if L == 1:                        # context length one returns the value row exactly
            assert np.array_equal(got[b], np.broadcast_to(case.v[b, 0].float().numpy(), (64, 256)))


def test_hint_larger_than_lengths_and_clamping():
    _announce("hint > lens, and lens > hint are clamped")
    case = W.make_contiguous_case("hint", 131, B=3, S=512, seq_lens=[100, 257, 512], poison=False)
    ctx = U.get_ctx()
    ref = U.run_oracle(case)
    got = U.run_gpu(ctx, case, hint=512)
    assert U.row_normalised_error(got, ref) <= U.TOL_BF16
    # a hint below a sequence's length truncates that sequence to the hint (documented behaviour)
    got2 = U.run_gpu(ctx, case, hint=256)
    trunc = W.make_contiguous_case("hint", 131, B=3, S=512, seq_lens=[100, 256, 256], poison=False)
    assert U.row_normalised_error(got2, U.run_oracle(trunc)) <= U.TOL_BF16


def test_single_split_path():
    """With one work item per sequence the kernel writes the final result itself (no merge pass)."""
    _announce("single split")
    ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=8, max_seq_len=2048, target_workgroups=1))
    assert mfa.mfa_decode_num_splits(ctx, 4, 1000) == 1
    case = W.make_contiguous_case("one", 141, B=4, S=1000, seq_lens=[1000, 1, 640, 0], poison=True)
    got = U.run_gpu(ctx, case)
    assert U.row_normalised_error(got, U.run_oracle(case)) <= U.TOL_BF16
    assert (got[3] == 0).all()
    ctx.close()


def test_many_splits_merge():
    """Few sequences, long context: every sequence is cut into many work items and merged."""
    _announce("many splits")
    ctx = U.get_ctx()
    case = W.make_contiguous_case("splits", 151, B=2, S=6000, seq_lens=[6000, 4321], poison=True)
    assert mfa.mfa_decode_num_splits(ctx, 2, 6000) > 16
    got = U.run_gpu(ctx, case)
    assert U.row_normalised_error(got, U.run_oracle(case)) <= U.TOL_BF16


def test_paged_equals_contiguous_bitwise_and_matches_oracle():
    _announce("paged vs contiguous")
    lens = [1, 64, 65, 200, 0, 127, 1000, 513]
    case = W.make_paged_case("paged", 161, lens, spare_pages=9, poison=True)
    contig = W.paged_to_contiguous(case, S=1024, poison=True)
    ctx = U.get_ctx()
    got_p = U.run_gpu(ctx, case, hint=1000)
    got_c = U.run_gpu(ctx, contig, hint=1000)
    assert np.array_equal(got_p, got_c)
    assert U.row_normalised_error(got_p, U.run_oracle(case)) <= U.TOL_BF16


def test_paged_gather_moves_bytes_exactly():
    _announce("paged gather memcmp")
    lens = [1, 64, 65, 200, 0, 127, 1000, 513]
    case = W.make_paged_case("gather", 162, lens, spare_pages=9, poison=False)
    contig = W.paged_to_contiguous(case, S=1024, poison=False)
    ctx = U.get_ctx()
    dst = torch.zeros(len(lens), 1024, 256, dtype=torch.bfloat16, device="cuda")
    mfa.mfa_debug_gather_paged(ctx, case.k_pool.cuda(), case.block_table.cuda(), case.seq_lens.cuda(), 1000, dst)
    torch.cuda.synchronize()
    got = dst.cpu().view(torch.int16)
    want = contig.k.view(torch.int16)
    for b, L in enumerate(lens):
        assert torch.equal(got[b, :L], want[b, :L])
        assert (got[b, L:] == 0).all()


def test_run_to_run_determinism():
    _announce("determinism")
    case = W.make_contiguous_case("det", 171, B=3, S=3000, seq_lens=[3000, 2999, 17], poison=True)
    ctx = U.get_ctx()
    a = U.run_gpu(ctx, case)
    b = U.run_gpu(ctx, case)
    assert np.array_equal(a, b)


def test_invariants_on_gpu_results():
    """Properties that hold at any size: zero query gives the mean value row; outputs are convex combinations."""
    _announce("invariants")
    case = W.make_contiguous_case("inv", 181, B=2, S=900, seq_lens=[900, 333], poison=True)
    case.q[0].zero_()
    ctx = U.get_ctx()
    got = U.run_gpu(ctx, case)
    v = case.v.float().numpy()
    mean0 = v[0, :900].astype(np.float64).mean(0)
    assert np.abs(got[0] - mean0).max() <= 1e-2 * np.abs(mean0).max()
    for b, L in enumerate([900, 333]):
        assert (got[b] <= v[b, :L].max(0) + 1e-5).all() and (got[b] >= v[b, :L].min(0) - 1e-5).all()


def test_argument_errors_through_the_c_abi():
    _announce("argument errors")
    ctx = U.get_ctx(max_batch=4, max_seq_len=1024)
    L = mfa.binding.lib()
    case = W.make_contiguous_case("err", 191, B=2, S=128, poison=False)
    q, k, v, lens = case.q.cuda(), case.k.cuda(), case.v.cuda(), case.seq_lens.cuda()
    out = torch.empty(2, 64, 256, device="cuda")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    call = lambda **kw: L.mfa_decode_attn(ctx.handle, kw.get("q", p(q)), p(k), p(v), kw.get("ks"), None,
                                          kw.get("dt", 0), kw.get("stride", 128), p(lens), kw.get("hint", 128),
                                          kw.get("B", 2), p(out), None)
    assert call() == mfa.MFA_OK
    assert call(q=None) == mfa.MFA_ERR_INVALID_ARG
    assert call(q=ctypes.c_void_p(q.data_ptr() + 2)) == mfa.MFA_ERR_INVALID_ARG     # misaligned
    assert call(B=0) == mfa.MFA_ERR_INVALID_ARG
    assert call(B=5) == mfa.MFA_ERR_INVALID_ARG                                     # > max_batch
    assert call(hint=0) == mfa.MFA_ERR_INVALID_ARG
    assert call(hint=2048) == mfa.MFA_ERR_INVALID_ARG                               # > max_seq_len
    assert call(stride=64) == mfa.MFA_ERR_INVALID_ARG                               # stride < hint
    assert call(dt=1) == mfa.MFA_ERR_INVALID_ARG                                    # fp8 without scales
    assert call(dt=7) == mfa.MFA_ERR_INVALID_ARG
    torch.cuda.synchronize()


def test_page_ids_outside_the_pool_touch_nothing_outside_it():
    """A block table with garbage ids for one sequence: reads are clamped into the pool (that sequence's result
    is meaningless), the other sequences are unaffected, and the append writes nothing for a bad id."""
    print("\n[case] bad page ids", flush=True)
    lens = [200, 130, 64, 300]
    case = W.make_paged_case("badids", 95, lens, spare_pages=3, poison=False)
    ref = U.run_oracle(case)
    bad = case.block_table.clone()
    bad[1, 0], bad[1, 1], bad[1, 2] = -7, 2 ** 30, case.k_pool.shape[0]
    ctx = U.get_ctx()
    d = U.to_dev
    out = mfa.mfa_decode_attn_paged(ctx, d(case.q), d(case.k_pool), d(case.v_pool), d(bad), d(case.seq_lens), 300)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    for b in (0, 2, 3):
        assert U.row_normalised_error(got[b], ref[b]) <= U.TOL_BF16
    # append: sequence 1's next row would land in page id 2**30 -> skipped; the others are written
    x = torch.randn(4, 7168, generator=torch.Generator().manual_seed(96)).to(torch.bfloat16)
    w_kv = (torch.randn(7168, 512, generator=torch.Generator().manual_seed(97)) * 0.02).to(torch.bfloat16)
    kp, vp = d(case.k_pool).clone(), d(case.v_pool).clone()
    before = kp.clone()
    at = torch.tensor([64, 64, 10, 70], dtype=torch.int32)       # row 0 of block 1, ..., block 1 of sequence 1 is the bad id
    mfa.mfa_kv_append_paged(ctx, d(x), d(w_kv), kp, vp, d(bad), d(at))
    torch.cuda.synchronize()
    changed = (kp != before).any(dim=2).cpu()                     # [n_pages, page]
    want = torch.zeros_like(changed)
    for b in (0, 2, 3):
        want[int(case.block_table[b, int(at[b]) // 64]), int(at[b]) % 64] = True
    assert torch.equal(changed, want)
