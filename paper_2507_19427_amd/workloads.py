"""Seeded synthetic inputs shaped like Step-3's decode workloads.

Input generation only: nothing here computes attention, softmax, a projection
or a normalisation.  The same host tensors feed the CPU oracle (as raw bit
patterns) and, copied to the device, the GPU library, so both sides see
identical bytes.  The paper's workloads are production traffic; these stand in
for their shapes: 64 query heads of dimension 256 over one shared key head and
one shared value head (Section 2), 64 sequences per GPU (Section 7.3, attention
latency table), contexts of 4K / 8K / 32K tokens (Sections 7.3), 64-token
cache pages.

Conventions
  * values are drawn as fp32 N(0,1) from torch.Generator(seed) in the order
    documented per function, then cast (round to nearest even) to storage;
  * cache memory past a sequence's length (rest of the last page, padding of
    the contiguous cache, spare pages) is filled with NaN when poison=True so
    that any read of it shows up in the result, and with finite values
    otherwise (timing runs);
  * fp8 caches are OCP e4m3fn codes with one fp32 scale per token per tensor:
    scale = max(|row|_inf, 1e-12) / 448, code = cast(row / scale).
"""
from dataclasses import dataclass, field
from typing import Optional

import torch

N_Q_HEADS = 64
HEAD_DIM = 256
D_MODEL = 7168
Q_RANK = 2048
PAGE_SIZE = 64
SOFTMAX_SCALE = 1.0 / 16.0
RMS_EPS = 1e-6
E4M3_MAX = 448.0


@dataclass
class AttnCase:
    """One decode-attention problem on the host."""
    name: str
    q: torch.Tensor                      # bf16 [B,H,D]
    seq_lens: torch.Tensor               # int32 [B]
    kv_dtype: str                        # "bf16" | "fp8" | "fp4" (e2m1, two per byte: [..., D/2] uint8)
    # contiguous cache
    k: Optional[torch.Tensor] = None     # [B,S,D]
    v: Optional[torch.Tensor] = None
    k_scale: Optional[torch.Tensor] = None   # fp32 [B,S]
    v_scale: Optional[torch.Tensor] = None
    # paged cache
    k_pool: Optional[torch.Tensor] = None    # [n_pages,page,D]
    v_pool: Optional[torch.Tensor] = None
    k_scale_pool: Optional[torch.Tensor] = None  # fp32 [n_pages,page]
    v_scale_pool: Optional[torch.Tensor] = None
    block_table: Optional[torch.Tensor] = None   # int32 [B,max_blocks]
    scale: float = SOFTMAX_SCALE
    extra: dict = field(default_factory=dict)

    @property
    def paged(self):
        return self.block_table is not None

    @property
    def B(self):
        return self.q.shape[0]

    @property
    def kv_tokens(self):
        return int(self.seq_lens.sum().item())


def _randn(gen, *shape):
    return torch.randn(*shape, generator=gen, dtype=torch.float32)


def quantize_e4m3_per_token(x):
    """fp32 [..., D] -> (e4m3fn codes [..., D], fp32 scales [...]) with one scale per row."""
    amax = x.abs().amax(dim=-1)
    scale = torch.clamp(amax, min=1e-12) / E4M3_MAX
    y = (x / scale.unsqueeze(-1)).clamp_(-E4M3_MAX, E4M3_MAX)
    return y.to(torch.float8_e4m3fn), scale.contiguous()


E2M1_MAX = 6.0


def quantize_e2m1_per_token(x):
    """fp32 [..., D] -> (e2m1 codes packed two per byte [..., D/2] uint8, fp32 scales [...]): one scale per
    row, nearest grid value with ties to the even code, element 2i in the low four bits of byte i."""
    amax = x.abs().amax(dim=-1)
    scale = torch.clamp(amax, min=1e-12) / E2M1_MAX
    y = (x / scale.unsqueeze(-1)).clamp_(-E2M1_MAX, E2M1_MAX)
    a = y.abs()
    code = torch.zeros_like(a, dtype=torch.uint8)
    # midpoints between neighbouring magnitudes 0, .5, 1, 1.5, 2, 3, 4, 6; a tie goes to the even code
    for mid, tie_goes_up in ((0.25, False), (0.75, True), (1.25, False), (1.75, True), (2.5, False), (3.5, True),
                             (5.0, False)):
        code += ((a >= mid) if tie_goes_up else (a > mid)).to(torch.uint8)
    code |= torch.signbit(y).to(torch.uint8) << 3
    packed = code[..., 0::2] | (code[..., 1::2] << 4)
    return packed.contiguous(), scale.contiguous()


def _nan_like(t):
    """A tensor of t's shape and dtype full of NaN codes (packed 4-bit codes have no NaN: all ones, and the
    scale beside them is NaN)."""
    if t.dtype == torch.uint8:
        return torch.full(t.shape, 0xFF, dtype=torch.uint8)
    if t.dtype == torch.float8_e4m3fn:
        return torch.full(t.shape, 0x7F, dtype=torch.uint8).view(torch.float8_e4m3fn)
    return torch.full(t.shape, float("nan"), dtype=t.dtype)


def _poison_contiguous(case: AttnCase):
    S = case.k.shape[1]
    for b in range(case.B):
        L = int(case.seq_lens[b])
        if L < S:
            for name in ("k", "v", "k_scale", "v_scale"):
                t = getattr(case, name)
                if t is not None:
                    t[b, L:] = _nan_like(t[b, L:])


def make_contiguous_case(name, seed, B, S, seq_lens=None, kv_dtype="bf16", poison=True,
                         H=N_Q_HEADS, D=HEAD_DIM, scale=SOFTMAX_SCALE) -> AttnCase:
    """Draw order: Q [B,H,D], K [B,S,D], V [B,S,D]."""
    gen = torch.Generator().manual_seed(seed)
    q = _randn(gen, B, H, D).to(torch.bfloat16)
    k32 = _randn(gen, B, S, D)
    v32 = _randn(gen, B, S, D)
    if seq_lens is None:
        seq_lens = [S] * B
    lens = torch.tensor(list(seq_lens), dtype=torch.int32)
    assert lens.shape == (B,) and int(lens.max()) <= S
    case = AttnCase(name=name, q=q, seq_lens=lens, kv_dtype=kv_dtype, scale=scale)
    if kv_dtype == "bf16":
        case.k, case.v = k32.to(torch.bfloat16), v32.to(torch.bfloat16)
    elif kv_dtype == "fp8":
        case.k, case.k_scale = quantize_e4m3_per_token(k32)
        case.v, case.v_scale = quantize_e4m3_per_token(v32)
    elif kv_dtype == "fp4":
        case.k, case.k_scale = quantize_e2m1_per_token(k32)
        case.v, case.v_scale = quantize_e2m1_per_token(v32)
    else:
        raise ValueError(kv_dtype)
    if poison:
        _poison_contiguous(case)
    return case


def make_multi_query(case: AttnCase, q_len, seed):
    """bf16 [B, q_len, H, D] queries for a step that decodes q_len tokens per sequence (the same
    distribution as the single query; the last of them is the case's own q)."""
    gen = torch.Generator().manual_seed(seed)
    B, H, D = case.q.shape
    extra = _randn(gen, B, q_len - 1, H, D).to(torch.bfloat16)
    return torch.cat([extra, case.q.unsqueeze(1)], dim=1).contiguous()


def make_paged_case(name, seed, seq_lens, kv_dtype="bf16", poison=True, spare_pages=64,
                    max_blocks=None, page=PAGE_SIZE, H=N_Q_HEADS, D=HEAD_DIM,
                    scale=SOFTMAX_SCALE) -> AttnCase:
    """Draw order: page permutation, K pool, V pool, Q.

    Logical block i of sequence b lives in page block_table[b, i]; the pages of all
    sequences are taken in order from a random permutation of the pool, unused table
    entries are -1.
    """
    gen = torch.Generator().manual_seed(seed)
    lens = torch.tensor(list(seq_lens), dtype=torch.int32)
    B = lens.numel()
    n_blocks = [(int(L) + page - 1) // page for L in lens]
    n_pages = sum(n_blocks) + spare_pages
    width = max_blocks if max_blocks is not None else max(max(n_blocks), 1)
    assert width >= max(n_blocks)
    perm = torch.randperm(n_pages, generator=gen).to(torch.int32)
    table = torch.full((B, width), -1, dtype=torch.int32)
    used = torch.zeros(n_pages, page, dtype=torch.bool)
    pos = 0
    for b in range(B):
        nb = n_blocks[b]
        ids = perm[pos:pos + nb]
        table[b, :nb] = ids
        pos += nb
        L = int(lens[b])
        for i in range(nb):
            used[int(ids[i]), : min(page, L - i * page)] = True
    k32 = _randn(gen, n_pages, page, D)
    v32 = _randn(gen, n_pages, page, D)
    q = _randn(gen, B, H, D).to(torch.bfloat16)
    case = AttnCase(name=name, q=q, seq_lens=lens, kv_dtype=kv_dtype, block_table=table, scale=scale)
    if kv_dtype == "bf16":
        case.k_pool, case.v_pool = k32.to(torch.bfloat16), v32.to(torch.bfloat16)
    elif kv_dtype == "fp8":
        case.k_pool, case.k_scale_pool = quantize_e4m3_per_token(k32)
        case.v_pool, case.v_scale_pool = quantize_e4m3_per_token(v32)
    elif kv_dtype == "fp4":
        case.k_pool, case.k_scale_pool = quantize_e2m1_per_token(k32)
        case.v_pool, case.v_scale_pool = quantize_e2m1_per_token(v32)
    else:
        raise ValueError(kv_dtype)
    if poison:
        for nm in ("k_pool", "v_pool", "k_scale_pool", "v_scale_pool"):
            t = getattr(case, nm)
            if t is not None:
                t[~used] = _nan_like(t[~used])
    case.extra["used_mask"] = used
    return case


def paged_to_contiguous(case: AttnCase, S=None, poison=True) -> AttnCase:
    """Gather a paged case into the equivalent contiguous cache (host copy; test helper)."""
    assert case.paged
    page = case.k_pool.shape[1]
    B = case.B
    S = S or max(int(case.seq_lens.max()), 1)
    D = case.k_pool.shape[2]
    out = AttnCase(name=case.name + "/contig", q=case.q, seq_lens=case.seq_lens,
                   kv_dtype=case.kv_dtype, scale=case.scale)
    out.k = _nan_like(torch.empty(B, S, D, dtype=case.k_pool.dtype)) if poison else torch.zeros(B, S, D, dtype=case.k_pool.dtype)
    out.v = out.k.clone()
    if case.kv_dtype != "bf16":
        out.k_scale = torch.full((B, S), float("nan") if poison else 1.0, dtype=torch.float32)
        out.v_scale = out.k_scale.clone()
    for b in range(B):
        L = int(case.seq_lens[b])
        for i in range((L + page - 1) // page):
            n = min(page, L - i * page)
            p = int(case.block_table[b, i])
            out.k[b, i * page:i * page + n] = case.k_pool[p, :n]
            out.v[b, i * page:i * page + n] = case.v_pool[p, :n]
            if case.kv_dtype != "bf16":
                out.k_scale[b, i * page:i * page + n] = case.k_scale_pool[p, :n]
                out.v_scale[b, i * page:i * page + n] = case.v_scale_pool[p, :n]
    return out


@dataclass
class QueryProjCase:
    """Inputs of the low-rank query path: x [B,d_model], W_qa [d_model,r], W_qb [r,H*D], all bf16."""
    name: str
    x: torch.Tensor
    w_qa: torch.Tensor
    w_qb: torch.Tensor
    gain: Optional[torch.Tensor] = None   # fp32 [r] or None (= unit gain)
    eps: float = RMS_EPS


def make_query_proj_case(name, seed, B, d_model=D_MODEL, r=Q_RANK, n_out=N_Q_HEADS * HEAD_DIM,
                         w_std=0.02, with_gain=False) -> QueryProjCase:
    """Draw order: x N(0,1), W_qa N(0,w_std^2), W_qb N(0,w_std^2), optional gain 1 + 0.1 N(0,1)."""
    gen = torch.Generator().manual_seed(seed)
    x = _randn(gen, B, d_model).to(torch.bfloat16)
    w_qa = (_randn(gen, d_model, r) * w_std).to(torch.bfloat16)
    w_qb = (_randn(gen, r, n_out) * w_std).to(torch.bfloat16)
    gain = (1.0 + 0.1 * _randn(gen, r)) if with_gain else None
    return QueryProjCase(name=name, x=x, w_qa=w_qa, w_qb=w_qb, gain=gain)


# ---------------------------------------------------------------------------
# The five named workloads.
# ---------------------------------------------------------------------------

def config1_tiny(poison=True):
    """Batch 2, context 256, contiguous bf16 (oracle-sized)."""
    return make_contiguous_case("cfg1_tiny", 1, B=2, S=256, poison=poison)


def config2_step3(poison=False):
    """Batch 64, context 4096 each, contiguous bf16: the throughput gate."""
    return make_contiguous_case("cfg2_b64_ctx4096", 2, B=64, S=4096, poison=poison)


def config3_lens(seed=3, B=128, lo=1024, hi=8192):
    gen = torch.Generator().manual_seed(seed)
    return torch.randint(lo, hi + 1, (B,), generator=gen, dtype=torch.int32)


def config3_ragged_paged(poison=True):
    """128 sequences, context uniform in [1024, 8192], 64-token pages, permuted block table."""
    lens = config3_lens()
    return make_paged_case("cfg3_ragged_paged", 3, lens.tolist(), poison=poison, spare_pages=64,
                           max_blocks=128)


def config4_long(poison=False):
    """Batch 16, context 32768 each, contiguous bf16: exercises the split/merge over the context."""
    return make_contiguous_case("cfg4_b16_ctx32768", 4, B=16, S=32768, poison=poison)


def config5_query():
    """x [128,7168] -> W_qa [7168,2048] -> RMSNorm -> W_qb [2048,16384]."""
    return make_query_proj_case("cfg5_query", 5, B=128)


def config5_fp8_cache(q, poison=False, seed=6):
    """fp8 e4m3 cache with per-token scales, batch 128, context 8192; q is supplied by the query path.

    Drawn per sequence (K row block then V row block) so the fp32 staging stays small.
    """
    B, S, D = 128, 8192, HEAD_DIM
    gen = torch.Generator().manual_seed(seed)
    k = torch.empty(B, S, D, dtype=torch.float8_e4m3fn)
    v = torch.empty(B, S, D, dtype=torch.float8_e4m3fn)
    ks = torch.empty(B, S, dtype=torch.float32)
    vs = torch.empty(B, S, dtype=torch.float32)
    for b in range(B):
        k[b], ks[b] = quantize_e4m3_per_token(_randn(gen, S, D))
        v[b], vs[b] = quantize_e4m3_per_token(_randn(gen, S, D))
    case = AttnCase(name="cfg5_fp8_b128_ctx8192", q=q, seq_lens=torch.full((B,), S, dtype=torch.int32),
                    kv_dtype="fp8", k=k, v=v, k_scale=ks, v_scale=vs)
    if poison:
        _poison_contiguous(case)
    return case
