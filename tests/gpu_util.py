"""Helpers shared by the GPU parity tests: move a host case to the device, run the library through
its binding, run the oracle on the same bytes, and compare with the row-normalised error."""
import numpy as np
import torch

import paper_2507_19427_amd as mfa
from oracle import mfa_oracle as O

TOL_BF16 = 1e-2      # max over rows of max_d|gpu-ref| / max_d|ref|, bf16 cache
TOL_FP8 = 3e-2       # same, fp8 and fp4 caches (the arithmetic after the codes is the same)

_ctx_cache = {}


def get_ctx(max_batch=128, max_seq_len=32768, **kw):
    key = (max_batch, max_seq_len, tuple(sorted(kw.items())))
    if key not in _ctx_cache:
        _ctx_cache[key] = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=max_batch, max_seq_len=max_seq_len, **kw))
    return _ctx_cache[key]


def to_dev(t):
    return None if t is None else t.cuda()


def run_gpu(ctx, case, hint=None):
    """Run one AttnCase through the C boundary; returns the fp32 output as a host numpy array."""
    hint = int(hint if hint is not None else max(int(case.seq_lens.max()), 1))
    q, lens = to_dev(case.q), to_dev(case.seq_lens)
    if case.paged:
        out = mfa.mfa_decode_attn_paged(ctx, q, to_dev(case.k_pool), to_dev(case.v_pool), to_dev(case.block_table),
                                        lens, hint, to_dev(case.k_scale_pool), to_dev(case.v_scale_pool))
    else:
        out = mfa.mfa_decode_attn(ctx, q, to_dev(case.k), to_dev(case.v), lens, hint, to_dev(case.k_scale),
                                  to_dev(case.v_scale))
    torch.cuda.synchronize()
    return out.cpu().numpy()


def run_oracle(case, rows=None):
    b = O.bits_of
    kd = {"bf16": O.KV_BF16, "fp8": O.KV_E4M3, "fp4": O.KV_E2M1}[case.kv_dtype]
    opt = lambda t: None if t is None else b(t)
    if case.paged:
        return O.decode_attn_paged(b(case.q), b(case.k_pool), b(case.v_pool), case.block_table.numpy(),
                                   case.seq_lens.numpy(), case.scale, k_scale_pool=opt(case.k_scale_pool),
                                   v_scale_pool=opt(case.v_scale_pool), kv_dtype=kd, rows=rows)
    return O.decode_attn(b(case.q), b(case.k), b(case.v), case.seq_lens.numpy(), case.scale,
                         k_scale=opt(case.k_scale), v_scale=opt(case.v_scale), kv_dtype=kd, rows=rows)


def row_normalised_error(got, ref):
    """max over rows of max_d|got-ref| / max_d|ref| (rows whose reference is all zero must match exactly)."""
    got = np.asarray(got, dtype=np.float64).reshape(-1, got.shape[-1])
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, ref.shape[-1])
    assert np.isfinite(got).all(), "non-finite values in the GPU result"
    num = np.abs(got - ref).max(axis=1)
    den = np.abs(ref).max(axis=1)
    zero = den == 0
    assert (num[zero] == 0).all()
    return float((num[~zero] / den[~zero]).max()) if (~zero).any() else 0.0


def sample_rows(case, n, seed=0, H=64):
    """n distinct (b,h) pairs, always including the first and last sequence and the longest one."""
    rng = np.random.default_rng(seed)
    B = case.B
    rows = {(0, 0), (B - 1, H - 1), (int(case.seq_lens.argmax()), 17), (int(case.seq_lens.argmin()), 40)}
    while len(rows) < n:
        rows.add((int(rng.integers(B)), int(rng.integers(H))))
    return sorted(rows)
