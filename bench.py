#!/usr/bin/env python3
"""Benchmark of the decode-step MFA attention on one MI355X.

Default workload (the one the metric is quoted on): batch 64, 64 query heads, one shared K/V head,
head dim 256, every sequence at context 4096, contiguous bf16 cache, synthetic N(0,1) values from a
fixed seed.  A step is one pass of the hot path over one batch: one mfa_decode_attn call (stream the
cache once, scores, online softmax, weighted sum, merge of the context splits); for the workload with
the query path, mfa_query_proj followed by the attention call.  Inputs are resident in HBM before the
timed region; the cache is rotated over several distinct buffer sets so that the 256 MB memory-side
cache cannot serve it.

--workload selects one of the other seeded workloads (ragged paged, long context, query path + fp8
cache, the whole attention layer at the paper's 8K / 32K contexts); they exist so that kernel profiles of
those shapes can be taken with this same program; cfg2q2 / fp8q2 run the step with two query tokens per
sequence, fp4 / fp4q2 the 4-bit cache.

Prints ONE JSON line: metric/value = KV tokens per second (from the wall time of exactly --steps steps), plus
  roofline      HBM roofline of the streaming attention kernel (`frac`: HIP events attached to that kernel's
                dispatch, EVENT_SAMPLES samples taken in a pass of their own right after the timed steps, whatever
                --steps is) and of the whole attention call, streaming kernel + merge kernel + the gap between
                them (`frac_whole_call`: from the wall time of the timed steps where a step is exactly that call;
                `frac_whole_call_by_events`: HIP events around the call on its stream, EVENT_SAMPLES samples, which
                cost the call about 2 us)
  cpu_baseline  the CPU oracle timed on this machine's host cores on a bounded sample of the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published peak
# HBM bytes per launch of the streaming kernel, NOT measured in this run: rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE (KiB per dispatch), each scaled by what the same counter reads for a 256 MiB device copy, as
# recorded in the named file under profiles/ (which gives the command and the library it was taken on).
PROFILED_TRAFFIC = {
    "cfg2": (132256 * 2.000 * 1024 + 16512 * 1.000 * 1024, "profiles/decode_attn_cfg2_b64_ctx4096_hbm_traffic.md"),
    "cfg4": (262560 * 2.000 * 1024 + 16512 * 1024, "profiles/decode_attn_other_workloads_hbm_traffic.md"),
    "cfg5": (276254 * 2.000 * 1024 + 16513 * 1024, "profiles/decode_attn_other_workloads_hbm_traffic.md"),
    "fp4": (140121 * 2.000 * 1024 + 16513 * 1024, "profiles/decode_attn_other_workloads_hbm_traffic.md"),
    "cfg2q2": (133280 * 2.000 * 1024 + 33024 * 1024, "profiles/decode_attn_other_workloads_hbm_traffic.md"),
    "cfg2q4": (135336 * 2.000 * 1024 + 66048 * 1024, "profiles/decode_attn_other_workloads_hbm_traffic.md"),
}
Q_BYTES_PER_SEQ = 64 * 256 * 2
OUT_BYTES_PER_SEQ = 64 * 256 * 4
EVENT_SAMPLES = 64                     # kernel-only and whole-call event samples, whatever --steps is
STREAM_READ_GRANULE = 2048 * 8192      # the plain-read probe takes multiples of this many bytes per buffer


class Workload:
    """What one step runs, and the figures the report needs."""
    def __init__(self):
        self.key = self.desc = self.metric = self.dtype = self.kernel = None
        self.steps = []            # one callable per buffer set
        self.read_pairs = []       # (K buffer, V buffer) per set for the plain-read reference, or empty
        self.T = 0                 # KV tokens per step
        self.kv_bytes_per_token = 0
        self.B = 0
        self.q_len = 1
        self.extra_config = {}
        self.case = None           # host case for the oracle sample
        self.attn_calls = []       # per buffer set: the attention call alone (equal to steps when the step is only that)
        self.attn_only = False
        self.keep = []


def _roll_sets(t, n_sets):
    import torch
    if t.element_size() == 1:                         # roll has no 8-bit float kernel: roll the bytes
        return [t] + [torch.roll(t.view(torch.uint8), shifts=i, dims=0).contiguous().view(t.dtype)
                      for i in range(1, n_sets)]
    return [t] + [torch.roll(t, shifts=i, dims=0).contiguous() for i in range(1, n_sets)]


def build_workload(key, mfa, W, n_sets):
    import torch
    w = Workload()
    w.key = key
    if key in ("cfg2", "cfg4"):
        case = W.config2_step3(poison=False) if key == "cfg2" else W.config4_long(poison=False)
        B, S = case.B, case.k.shape[1]
        w.ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=B, max_seq_len=S))
        q, lens = case.q.cuda(), case.seq_lens.cuda()
        ks, vs = _roll_sets(case.k.cuda(), n_sets), _roll_sets(case.v.cuda(), n_sets)
        out = torch.empty(B, 64, 256, dtype=torch.float32, device="cuda")
        # one prepared call per buffer set: the timed loop only crosses the C boundary
        w.steps = [mfa.PreparedDecodeAttn(w.ctx, q, ks[j], vs[j], lens, S, out) for j in range(n_sets)]
        w.read_pairs = list(zip(ks, vs))
        w.desc = ("configs[%d]: B=%d, 64 q heads, 1 shared K/V head, head_dim 256, ctx %d, contiguous bf16 KV"
                  % (1 if key == "cfg2" else 3, B, S))
        w.metric = "KV tokens/s, MFA decode attention, B=%d, ctx %d, bf16, 1 GPU" % (B, S)
        w.dtype, w.kernel, w.kv_bytes_per_token = "bf16", "mfa::decode_bf16_kernel<false, 1>", 1024
        w.T, w.B, w.case = case.kv_tokens, B, case
        w.attn_calls, w.attn_only = w.steps, True
        w.extra_config = {"n_splits": mfa.mfa_decode_num_splits(w.ctx, B, S)}
    elif key == "cfg3":
        case = W.config3_ragged_paged(poison=False)
        B, S = case.B, int(case.seq_lens.max())
        w.ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=B, max_seq_len=8192))
        q, lens, table = case.q.cuda(), case.seq_lens.cuda(), case.block_table.cuda()
        kp, vp = case.k_pool.cuda(), case.v_pool.cuda()
        ks = [kp] + [kp.clone() for _ in range(1, n_sets)]     # same pages and table, distinct memory
        vs = [vp] + [vp.clone() for _ in range(1, n_sets)]
        out = torch.empty(B, 64, 256, dtype=torch.float32, device="cuda")
        w.steps = [(lambda j=j: mfa.mfa_decode_attn_paged(w.ctx, q, ks[j], vs[j], table, lens, S, out=out))
                   for j in range(n_sets)]
        w.desc = ("configs[2]: B=128, ctx uniform in [1024, 8192], 64-token pages behind a permuted block table, "
                  "bf16 KV")
        w.metric = "KV tokens/s, MFA decode attention, B=128, ragged paged ctx 1K-8K, bf16, 1 GPU"
        w.dtype, w.kernel, w.kv_bytes_per_token = "bf16", "mfa::decode_bf16_kernel<true, 1>", 1024
        w.T, w.B, w.case = case.kv_tokens, B, case
        w.attn_calls, w.attn_only = w.steps, True
        w.extra_config = {"n_splits": mfa.mfa_decode_num_splits(w.ctx, B, S), "max_ctx": S}
    elif key == "cfg5":
        qc = W.config5_query()
        B = qc.x.shape[0]
        w.ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=B, max_seq_len=8192))
        x, w_qa, w_qb = qc.x.cuda(), qc.w_qa.cuda(), qc.w_qb.cuda()
        q = mfa.mfa_query_proj(w.ctx, x, w_qa, w_qb)
        case = W.config5_fp8_cache(q.cpu(), poison=False)
        S = case.k.shape[1]
        lens = case.seq_lens.cuda()
        ks, vs = _roll_sets(case.k.cuda(), n_sets), _roll_sets(case.v.cuda(), n_sets)
        kss, vss = _roll_sets(case.k_scale.cuda(), n_sets), _roll_sets(case.v_scale.cuda(), n_sets)
        out = torch.empty(B, 64, 256, dtype=torch.float32, device="cuda")
        attn = [mfa.PreparedDecodeAttn(w.ctx, q, ks[j], vs[j], lens, S, out, k_scale=kss[j], v_scale=vss[j])
                for j in range(n_sets)]

        def step(j):
            mfa.mfa_query_proj(w.ctx, x, w_qa, w_qb, q_out=q)
            attn[j]()
        w.steps = [(lambda j=j: step(j)) for j in range(n_sets)]
        w.read_pairs = list(zip(ks, vs))
        w.desc = ("configs[4]: B=128, query path 7168 -> 2048 -> RMSNorm -> 64x256, then attention over ctx 8192 of "
                  "fp8 e4m3 KV with per-token fp32 scales")
        w.metric = "KV tokens/s, MFA query path + decode attention, B=128, ctx 8192, fp8 KV, 1 GPU"
        w.dtype, w.kernel, w.kv_bytes_per_token = "bf16 (fp8 e4m3 KV storage)", "mfa::decode_lowbit_kernel<false, 1, 8>", 520
        w.T, w.B, w.case = case.kv_tokens, B, case
        w.attn_calls = attn
        w.extra_config = {"n_splits": mfa.mfa_decode_num_splits(w.ctx, B, S)}
        w.keep = [x, w_qa, w_qb]
    elif key in ("fp4", "fp4q2"):
        # 4-bit cache (Section 5.2: 4-bit storage, 8-bit arithmetic): the cache shape of configs[4] in e2m1
        # codes, 264 bytes per token with the two fp32 scales.
        case = W.make_contiguous_case(key, 6, B=128, S=8192, kv_dtype="fp4", poison=False)
        B, S = case.B, case.k.shape[1]
        q_len = 2 if key == "fp4q2" else 1
        w.ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=B, max_seq_len=S))
        q = (W.make_multi_query(case, 2, 9) if q_len == 2 else case.q).cuda()
        lens = case.seq_lens.cuda()
        ks, vs = _roll_sets(case.k.cuda(), n_sets), _roll_sets(case.v.cuda(), n_sets)
        kss, vss = _roll_sets(case.k_scale.cuda(), n_sets), _roll_sets(case.v_scale.cuda(), n_sets)
        out = torch.empty(*q.shape, dtype=torch.float32, device="cuda")
        w.steps = [mfa.PreparedDecodeAttn(w.ctx, q, ks[j], vs[j], lens, S, out, k_scale=kss[j], v_scale=vss[j])
                   for j in range(n_sets)]
        w.read_pairs = list(zip(ks, vs))
        w.desc = ("B=%d, 64 q heads, 1 shared K/V head, head_dim 256, ctx %d, contiguous 4-bit e2m1 KV with per-token "
                  "fp32 scales, %d query token(s) per sequence" % (B, S, q_len))
        w.metric = "KV tokens/s, MFA decode attention%s, B=%d, ctx %d, fp4 KV, 1 GPU" % (
            " with 2 query tokens" if q_len == 2 else "", B, S)
        w.dtype = "bf16 (fp4 e2m1 KV storage, e4m3 score arithmetic)"
        w.kernel = "mfa::decode_lowbit_kernel<false, %d, 4>" % q_len
        w.kv_bytes_per_token = 264
        w.T, w.B, w.q_len = case.kv_tokens, B, q_len
        w.attn_calls, w.attn_only = w.steps, True
        if q_len == 1:
            w.case = case
        w.extra_config = {"query_tokens_per_sequence": q_len}
    elif key in ("cfg2q2", "cfg2q3", "cfg2q4", "fp8q2"):
        # Several new tokens per sequence in one pass over the cache (the multi-token step of Section 5.2):
        # same cache shapes as configs[1] / the cache of configs[4], q_len times the arithmetic per byte.
        fp8 = key == "fp8q2"
        q_len = int(key[-1])
        case = (W.make_contiguous_case(key, 6, B=128, S=8192, kv_dtype="fp8", poison=False) if fp8
                else W.config2_step3(poison=False))
        B, S = case.B, case.k.shape[1]
        w.ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=B, max_seq_len=S))
        q, lens = W.make_multi_query(case, q_len, 9).cuda(), case.seq_lens.cuda()
        ks, vs = _roll_sets(case.k.cuda(), n_sets), _roll_sets(case.v.cuda(), n_sets)
        kss = _roll_sets(case.k_scale.cuda(), n_sets) if fp8 else [None] * n_sets
        vss = _roll_sets(case.v_scale.cuda(), n_sets) if fp8 else [None] * n_sets
        out = torch.empty(B, q_len, 64, 256, dtype=torch.float32, device="cuda")
        w.steps = [mfa.PreparedDecodeAttn(w.ctx, q, ks[j], vs[j], lens, S, out, k_scale=kss[j], v_scale=vss[j])
                   for j in range(n_sets)]
        w.read_pairs = list(zip(ks, vs))
        w.desc = ("%d query tokens per sequence: B=%d, 64 q heads, 1 shared K/V head, head_dim 256, ctx %d, "
                  "contiguous %s KV" % (q_len, B, S, "fp8 e4m3 (per-token fp32 scales)" if fp8 else "bf16"))
        w.metric = "KV tokens/s, MFA decode attention with %d query tokens, B=%d, ctx %d, %s, 1 GPU" % (
            q_len, B, S, "fp8 KV" if fp8 else "bf16")
        w.dtype = "bf16 (fp8 e4m3 KV storage)" if fp8 else "bf16"
        w.kernel = ("mfa::decode_lowbit_kernel<false, 2, 8>" if fp8 else
                    "mfa::decode_bf16_kernel<false, 2>" if q_len == 2 else "mfa::decode_bf16_multi_kernel<false, %d>" % q_len)
        w.kv_bytes_per_token = 520 if fp8 else 1024
        w.T, w.B, w.q_len = case.kv_tokens, B, q_len
        w.attn_calls, w.attn_only = w.steps, True
        w.extra_config = {"query_tokens_per_sequence": q_len}
    elif key in ("layer8k", "layer32k", "layer8k_fp8", "layer32k_fp8"):
        # One whole attention layer of a decode step, the unit of the paper's attention-latency table
        # (Section 7.3: 64 sequences per GPU, context 8K / 32K): query path, key/value projection of the
        # new token and its cache record, attention over the lengthened cache, output projection.
        # The _fp8 workloads keep the cache in e4m3 with per-token scales, as the paper's deployment does
        # (its linears are 8-bit too; ours stay bf16).
        fp8 = key.endswith("_fp8")
        S = 8192 if key.startswith("layer8k") else 32768
        B = 64
        case = W.make_contiguous_case(key, 7, B=B, S=S, kv_dtype="fp8" if fp8 else "bf16", poison=False)
        qc = W.make_query_proj_case(key + "_q", 5, B=B)
        gen = torch.Generator().manual_seed(8)
        w_kv = (torch.randn(W.D_MODEL, 2 * W.HEAD_DIM, generator=gen) * 0.02).to(torch.bfloat16)
        w_o = (torch.randn(W.N_Q_HEADS * W.HEAD_DIM, W.D_MODEL, generator=gen) * 0.02).to(torch.bfloat16)
        w.ctx = mfa.mfa_decode_init(mfa.MfaConfig(max_batch=B, max_seq_len=S))
        x = qc.x.cuda()
        ks, vs = _roll_sets(case.k.cuda(), n_sets), _roll_sets(case.v.cuda(), n_sets)
        kss = _roll_sets(case.k_scale.cuda(), n_sets) if fp8 else [None] * n_sets
        vss = _roll_sets(case.v_scale.cuda(), n_sets) if fp8 else [None] * n_sets
        # every layer of a model has its own weights: rotate them like the cache
        wsets = [tuple(t.cuda() if j == 0 else t.cuda().clone() for t in (qc.w_qa, qc.w_qb, w_kv, w_o)) for j in range(n_sets)]
        old_lens = torch.full((B,), S - 1, dtype=torch.int32, device="cuda")
        new_lens = torch.full((B,), S, dtype=torch.int32, device="cuda")
        q = torch.empty(B, 64, 256, dtype=torch.bfloat16, device="cuda")
        out = torch.empty(B, 64, 256, dtype=torch.float32, device="cuda")
        y = torch.empty(B, W.D_MODEL, dtype=torch.bfloat16, device="cuda")
        attn = [mfa.PreparedDecodeAttn(w.ctx, q, ks[j], vs[j], new_lens, S, out, k_scale=kss[j], v_scale=vss[j])
                for j in range(n_sets)]

        def step(j):
            wa, wb, wkv, wo = wsets[j]
            mfa.mfa_query_proj(w.ctx, x, wa, wb, q_out=q)
            mfa.mfa_kv_append(w.ctx, x, wkv, ks[j], vs[j], old_lens, k_scale=kss[j], v_scale=vss[j])
            attn[j]()
            mfa.mfa_out_proj(w.ctx, out, wo, y=y)
        w.steps = [(lambda j=j: step(j)) for j in range(n_sets)]
        w.read_pairs = list(zip(ks, vs))
        kv_name = "fp8 e4m3 KV with per-token scales" if fp8 else "bf16 KV"
        w.desc = ("attention layer of one decode step: B=64, query path 7168 -> 2048 -> 64x256, key/value projection "
                  "7168 -> 2x256 + cache record, attention over ctx %d of contiguous %s, output projection "
                  "16384 -> 7168; all weights bf16" % (S, kv_name))
        w.metric = "KV tokens/s, MFA attention layer (linears + core attention), B=64, ctx %d, %s, 1 GPU" % (
            S, "fp8 KV" if fp8 else "bf16")
        w.dtype = "bf16 (fp8 e4m3 KV storage)" if fp8 else "bf16"
        w.kernel = "mfa::decode_lowbit_kernel<false, 1, 8>" if fp8 else "mfa::decode_bf16_kernel<false, 1>"
        w.kv_bytes_per_token = 520 if fp8 else 1024
        w.T, w.B = B * S, B
        w.attn_calls = attn
        w.extra_config = {"n_splits": mfa.mfa_decode_num_splits(w.ctx, B, S),
                          "weight_bytes_per_step": 2 * (qc.w_qa.numel() + qc.w_qb.numel() + w_kv.numel() + w_o.numel()),
                          "paper_layer_time_us": {"ctx": S, "H800": 281 if S == 8192 else 791, "H20": 438 if S == 8192 else 1452,
                                                  "A800": 531 if S == 8192 else 1484,
                                                  "note": "attention-latency table of Section 7.3 (8-bit cache and 8-bit "
                                                          "weights in the linears there)"}}
        w.keep = [x, wsets]
    else:
        raise ValueError(key)
    return w


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", choices=("cfg2", "cfg3", "cfg4", "cfg5", "cfg2q2", "cfg2q3", "cfg2q4", "fp8q2", "fp4", "fp4q2", "layer8k", "layer32k", "layer8k_fp8", "layer32k_fp8"), default="cfg2")
    ap.add_argument("--buffer-sets", type=int, default=None, help="distinct KV buffer sets rotated through")
    ap.add_argument("--settle-ms", type=float, default=40.0,
                    help="run untimed steps for this long before the --warmup steps: the device reaches its steady clocks "
                         "only after some tens of milliseconds of load (first ~20 ms: steps 2-7 %% slower)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU work for the oracle sample")
    ap.add_argument("--calibration-copy", type=int, default=0, metavar="N",
                    help="after the timed steps, run N device-to-device copies of 256 MiB: a kernel of known HBM "
                         "traffic beside which rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU's share of the data-parallel decode path; "
              "--gpus above 1 is not supported (every GPU would run this same kernel on its own sequences).",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2507_19427_amd as mfa
    from paper_2507_19427_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    n_sets = max(1, args.buffer_sets if args.buffer_sets is not None else (5 if args.workload == "cfg2" else 3))
    w = build_workload(args.workload, mfa, W, n_sets)
    ctx, T = w.ctx, w.T

    # A decode loop runs for seconds; a benchmark of 20 steps lasts a millisecond.  Untimed steps until the device
    # has been under load for --settle-ms, then the W warm-up steps asked for.
    n_settle = 0
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(16):
            w.steps[n_settle % n_sets]()
            n_settle += 1
        torch.cuda.synchronize()
    for i in range(args.warmup):
        w.steps[i % n_sets]()
    torch.cuda.synchronize()

    # The timed region: exactly K steps, nothing attached to them, barrier-free on one GPU
    # (synchronize on both sides).
    K = args.steps
    t0 = time.perf_counter()
    for i in range(K):
        w.steps[i % n_sets]()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K

    # Roofline samples, in a pass of their own right after the timed steps (same buffers, same rotation):
    # (1) HIP events attached by the library to the dispatch of the streaming kernel, on the stream the kernel
    #     is launched on: the duration of that kernel alone (a dispatch that carries events costs the step
    #     about 3.5 us of wall time, which is why the timed steps above carry none);
    # (2) HIP events recorded on that stream around the whole attention call, i.e. streaming kernel + merge
    #     kernel + the gap between them: the t of "KV tokens / t" for one call.
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(EVENT_SAMPLES)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(EVENT_SAMPLES)]
    for e in starts + stops:
        e.record()                                   # materialise the HIP event handles
    torch.cuda.synchronize()
    for i in range(EVENT_SAMPLES):
        mfa.mfa_debug_set_kernel_events(ctx, starts[i], stops[i])
        w.steps[i % n_sets]()
    torch.cuda.synchronize()
    mfa.mfa_debug_set_kernel_events(ctx, None, None)
    ev_ms = sorted(s.elapsed_time(e) for s, e in zip(starts, stops))
    ev_mean = sum(ev_ms) / len(ev_ms)
    ev_median = ev_ms[len(ev_ms) // 2]
    call_ms = None
    if w.attn_calls:
        for i in range(EVENT_SAMPLES):
            starts[i].record()
            w.attn_calls[i % n_sets]()
            stops[i].record()
        torch.cuda.synchronize()
        call_ms = sorted(s.elapsed_time(e) for s, e in zip(starts, stops))

    if args.calibration_copy > 0:
        src = torch.randint(0, 255, (256 << 20,), dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.calibration_copy):
            dst.copy_(src)
        torch.cuda.synchronize()

    value = T / (ms_per_step * 1e-3)
    algo_bytes = T * w.kv_bytes_per_token + w.B * w.q_len * (Q_BYTES_PER_SEQ + OUT_BYTES_PER_SEQ)
    achieved = algo_bytes / (ev_mean * 1e-3) / 1e9
    traffic, traffic_source = PROFILED_TRAFFIC.get(w.key, (None, None))
    roofline = {
        "bound": "hbm",
        "kernel": w.kernel + " (HIP events recorded around it inside the attention call)",
        "achieved": achieved,
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS,
        "traffic": traffic,
        "traffic_source": traffic_source and (traffic_source + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a "
                                              "256 MiB copy; not measured in this run)"),
        "algorithmic_bytes_per_launch": algo_bytes,
        "event_ms_mean": ev_mean,
        "event_ms_median": ev_median,
        "event_ms_min": ev_ms[0],
        "event_samples": len(ev_ms),
    }
    if call_ms:
        call_median = call_ms[len(call_ms) // 2]
        roofline["whole_call"] = {
            "what": "one attention call = streaming kernel + merge kernel + the gap between them, HIP events "
                    "around the call on its stream",
            "ms_median": call_median, "ms_mean": sum(call_ms) / len(call_ms), "ms_min": call_ms[0],
            "samples": len(call_ms),
            "kv_tokens_per_s": T / (call_median * 1e-3),
        }
        roofline["frac_whole_call_by_events"] = algo_bytes / (call_median * 1e-3) / 1e9 / HBM_PEAK_GBS
        roofline["frac_whole_call"] = roofline["frac_whole_call_by_events"]
    if w.attn_only:
        # The step is exactly the attention call, so the wall time of the timed steps is the t of "KV tokens / t"
        # with nothing added: the pair of events around a call costs the call about 2 us.  This is the figure
        # reported as frac_whole_call for these workloads.
        roofline["frac_whole_call_from_ms_per_step"] = algo_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS
        roofline["frac_whole_call"] = roofline["frac_whole_call_from_ms_per_step"]

    # Reference: a do-nothing kernel that only reads the same K and V buffers (plain 16-byte loads), timed
    # the same way.  It bounds what any kernel streaming these bytes can reach on this device.
    if w.read_pairs:
        nbytes = w.read_pairs[0][0].numel() * w.read_pairs[0][0].element_size()
        if nbytes % STREAM_READ_GRANULE == 0:
            n_ref = min(len(starts), EVENT_SAMPLES)
            for i in range(3):
                mfa.mfa_debug_stream_read(ctx, *w.read_pairs[i % n_sets])
            torch.cuda.synchronize()
            for i in range(n_ref):
                mfa.mfa_debug_set_kernel_events(ctx, starts[i], stops[i])
                mfa.mfa_debug_stream_read(ctx, *w.read_pairs[i % n_sets])
            torch.cuda.synchronize()
            mfa.mfa_debug_set_kernel_events(ctx, None, None)
            ref_ms = sum(s.elapsed_time(e) for s, e in zip(starts[:n_ref], stops[:n_ref])) / n_ref
            ref_gbs = 2 * nbytes / (ref_ms * 1e-3) / 1e9
            kv_gbs = 2 * nbytes / (ev_mean * 1e-3) / 1e9
            roofline["plain_read_of_same_kv"] = {
                "GBps": ref_gbs, "ms": ref_ms, "frac_of_peak": ref_gbs / HBM_PEAK_GBS,
                "note": "do-nothing kernel reading the same K,V buffers once; attention kernel's rate over those "
                        "bytes / this = %.3f" % (kv_gbs / ref_gbs)}

    cfg = {"workload": w.desc, "kv_tokens_per_step": T, "kv_buffer_sets": n_sets,
           "settle_ms_before_warmup": args.settle_ms, "settle_steps": n_settle}
    cfg.update(w.extra_config)
    result = {
        "metric": w.metric,
        "value": value,
        "unit": "KV tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": cfg,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w.case, args.cpu_seconds) if w.case is not None else None
    print(json.dumps(result), flush=True)
    ctx.close()


def cpu_baseline(case, target_seconds):
    """Time the CPU oracle, as it stands, on a bounded sample of the same workload: whole sequences (all 64
    heads) from the front of the batch, as many as fit the time budget (one (sequence, head) row is the
    oracle's unit of work; its rows run on all host threads).  Also timed: one sequence on a single thread."""
    from oracle import mfa_oracle as O
    b = O.bits_of
    threads = O.get_threads()
    kd = {"bf16": O.KV_BF16, "fp8": O.KV_E4M3, "fp4": O.KV_E2M1}[case.kv_dtype]
    opt = lambda t: None if t is None else b(t)
    lens = case.seq_lens.numpy()

    def run(n_seq):
        rows = [(i, h) for i in range(n_seq) for h in range(64)]
        t0 = time.perf_counter()
        if case.paged:
            O.decode_attn_paged(b(case.q), b(case.k_pool), b(case.v_pool), case.block_table.numpy(), lens, case.scale,
                                k_scale_pool=opt(case.k_scale_pool), v_scale_pool=opt(case.v_scale_pool), kv_dtype=kd,
                                rows=rows)
        else:
            O.decode_attn(b(case.q), b(case.k), b(case.v), lens, case.scale, k_scale=opt(case.k_scale),
                          v_scale=opt(case.v_scale), kv_dtype=kd, rows=rows)
        return time.perf_counter() - t0

    t1 = run(1)                                        # calibration: one sequence, all 64 heads
    per_token = t1 / max(int(lens[0]), 1)
    n, tok = 1, int(lens[0])
    while n < case.B and (tok + int(lens[n])) * per_token <= target_seconds:
        tok += int(lens[n])
        n += 1
    t = run(n) if n > 1 else t1
    tokens = int(lens[:n].sum())
    O.set_threads(1)
    try:
        t_single = run(1)
    finally:
        O.set_threads(threads)
    return {
        "value": tokens / t,
        "unit": "KV tokens/s",
        "cores": threads,
        "kind": "oracle",
        "sample": f"first {n} of {case.B} sequences of the same workload (all 64 heads, {tokens} KV tokens) in {t:.2f} s",
        "single_thread": {"value": int(lens[0]) / t_single, "unit": "KV tokens/s", "cores": 1,
                          "sample": f"the first sequence (all 64 heads, {int(lens[0])} KV tokens) in {t_single:.2f} s"},
    }


if __name__ == "__main__":
    main()
