"""Seeded random sweep through the C-ABI: ragged batches of several shapes (all short, a few very long among
short ones, uniform, with empty sequences), every cache type, contiguous and paged, one to four query tokens,
hints above the longest length.  Each case is compared with the oracle at the usual tolerances; the point is the
combinations that the hand-picked cases of the other files do not list."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2507_19427_amd as mfa
from paper_2507_19427_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _one_case(rng, i, ctx):
    kv = ["bf16", "fp8", "fp4"][i % 3]
    B = int(rng.choice([1, 2, 3, 7, 16, 33, 64, 100, 257, 400]))
    style = int(rng.integers(0, 4))
    if style == 0:
        lens = rng.integers(0, 130, B)
    elif style == 1:
        lens = rng.integers(1, 2000 if B <= 33 else 300, B)
    elif style == 2:
        lens = np.where(rng.random(B) < 0.1, rng.integers(1000, 6000 if B <= 16 else 1200), rng.integers(0, 70, B))
    else:
        lens = np.full(B, int(rng.integers(1, 700)))
    lens = [int(x) for x in lens]
    q_len = int(rng.choice([1, 1, 2, 3, 4]))
    paged = bool(rng.integers(0, 2))
    seed = int(rng.integers(1, 1 << 30))
    S = max(max(lens), 1) + int(rng.integers(0, 9))
    if paged:
        case = W.make_paged_case("sweep", seed, lens, kv_dtype=kv, spare_pages=int(rng.integers(0, 6)), poison=True)
    else:
        case = W.make_contiguous_case("sweep", seed, B=B, S=S, seq_lens=lens, kv_dtype=kv, poison=True)
    hint = max(max(lens), 1) + int(rng.integers(0, 3)) * 64
    hint = min(hint, S) if not paged else min(hint, case.block_table.shape[1] * 64)
    tol = U.TOL_BF16 if kv == "bf16" else U.TOL_FP8
    print(f"   case {i}: kv={kv} B={B} q_len={q_len} paged={int(paged)} style={style} longest={max(lens)} hint={hint}",
          flush=True)
    d = U.to_dev
    if q_len == 1:
        got, ref = U.run_gpu(ctx, case, hint=hint), U.run_oracle(case)
    else:
        qm = W.make_multi_query(case, q_len, seed + 1)
        if paged:
            out = mfa.mfa_decode_attn_paged_multi(ctx, d(qm), d(case.k_pool), d(case.v_pool), d(case.block_table),
                                                  d(case.seq_lens), hint, d(case.k_scale_pool), d(case.v_scale_pool))
        else:
            out = mfa.mfa_decode_attn_multi(ctx, d(qm), d(case.k), d(case.v), d(case.seq_lens), hint, d(case.k_scale),
                                            d(case.v_scale))
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        ref = np.stack([U.run_oracle(dataclasses.replace(
            case, q=qm[:, j].contiguous(), seq_lens=torch.clamp(case.seq_lens - (q_len - 1 - j), min=0).to(torch.int32)))
            for j in range(q_len)], axis=1)
    err = U.row_normalised_error(got, ref)
    assert err <= tol, (i, err)
    return err / tol


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_sweep(seed):
    print(f"\n[case] random sweep, seed {seed}", flush=True)
    rng = np.random.default_rng(seed)
    ctx = U.get_ctx(max_batch=512, max_seq_len=8192)
    worst = max(_one_case(rng, i, ctx) for i in range(15))
    print(f"   worst error as a fraction of the tolerance: {worst:.2f}", flush=True)
