"""GPU parity for the pieces of the attention layer around the core: the key/value projection of the new
token with its cache record (bf16 rounding or per-token e4m3 quantisation, contiguous or paged), and the
output projection.

The record step is integer/byte work decided by floating point: given the same fp32 rows it must agree with
the oracle's single-precision quantiser bit for bit (codes, scales, bf16 patterns).  The projections are
compared with the oracle's fp64 product within a tolerance; end to end, the stored record must be the
oracle's record of a row that lies within that tolerance of the fp64 projection."""
import numpy as np
import pytest
import torch

import paper_2507_19427_amd as mfa
from paper_2507_19427_amd import workloads as W
from oracle import mfa_oracle as O

import gpu_util as U

pytestmark = pytest.mark.gpu

TOL_LINEAR = 1e-2     # row-normalised, bf16 storage of the result (and of the activations for the output projection)


def _rows_kv(seed, B, scale_rows=True):
    g = torch.Generator().manual_seed(seed)
    kv = torch.randn(B, 512, generator=g)
    if scale_rows:
        kv *= torch.logspace(-6, 6, B).unsqueeze(1)           # rows of very different magnitude
    if B > 3:
        kv[2] = 0.0                                           # an all-zero row: scale floor
        kv[3, :256] = 1e-30                                   # below the floor
    return kv


@pytest.mark.parametrize("paged", [False, True])
def test_record_is_bit_exact_fp8(paged):
    print(f"\n[case] kv record fp8 paged={paged}", flush=True)
    B = 37
    kv = _rows_kv(401, B)
    lens = torch.tensor([(7 * b) % 130 for b in range(B)], dtype=torch.int32)
    ctx = U.get_ctx()
    codes_k, scale_k = O.quantize_rows_e4m3(kv[:, :256].numpy())
    codes_v, scale_v = O.quantize_rows_e4m3(kv[:, 256:].numpy())
    if paged:
        n_pages, width = 3 * B + 5, 3
        g = torch.Generator().manual_seed(402)
        perm = torch.randperm(n_pages, generator=g).to(torch.int32)
        table = perm[:B * width].reshape(B, width).contiguous()
        k = torch.full((n_pages, 64, 256), 0x55, dtype=torch.uint8).cuda()
        v = torch.full((n_pages, 64, 256), 0x55, dtype=torch.uint8).cuda()
        ks = torch.full((n_pages, 64), -1.0).cuda()
        vs = torch.full((n_pages, 64), -1.0).cuda()
        mfa.mfa_debug_kv_record(ctx, kv.cuda(), k.view(torch.float8_e4m3fn), v.view(torch.float8_e4m3fn), lens.cuda(),
                                ks, vs, block_table=table.cuda())
        rows = [(int(table[b, int(lens[b]) // 64]), int(lens[b]) % 64) for b in range(B)]
    else:
        S = 131
        k = torch.full((B, S, 256), 0x55, dtype=torch.uint8).cuda()
        v = torch.full((B, S, 256), 0x55, dtype=torch.uint8).cuda()
        ks = torch.full((B, S), -1.0).cuda()
        vs = torch.full((B, S), -1.0).cuda()
        mfa.mfa_debug_kv_record(ctx, kv.cuda(), k.view(torch.float8_e4m3fn), v.view(torch.float8_e4m3fn), lens.cuda(), ks, vs)
        rows = [(b, int(lens[b])) for b in range(B)]
    torch.cuda.synchronize()
    k, v, ks, vs = k.cpu().numpy(), v.cpu().numpy(), ks.cpu().numpy(), vs.cpu().numpy()
    touched = np.zeros(k.shape[:2], dtype=bool)
    for b, (i, j) in enumerate(rows):
        assert np.array_equal(k[i, j], codes_k[b]) and np.array_equal(v[i, j], codes_v[b]), b
        assert ks[i, j] == scale_k[b] and vs[i, j] == scale_v[b], b
        touched[i, j] = True
    assert (k[~touched] == 0x55).all() and (v[~touched] == 0x55).all()          # nothing else was written
    assert (ks[~touched] == -1.0).all() and (vs[~touched] == -1.0).all()


def test_record_is_bit_exact_bf16_and_skips_rows_outside_the_cache():
    print("\n[case] kv record bf16", flush=True)
    B, S = 9, 40
    kv = _rows_kv(403, B)
    lens = torch.tensor([0, 39, 40, 17, 5, 100, 1, 38, 39], dtype=torch.int32)     # 40 and 100 lie outside
    ctx = U.get_ctx()
    k = torch.zeros(B, S, 256, dtype=torch.bfloat16).cuda()
    v = torch.zeros(B, S, 256, dtype=torch.bfloat16).cuda()
    mfa.mfa_debug_kv_record(ctx, kv.cuda(), k, v, lens.cuda())
    torch.cuda.synchronize()
    kb = k.cpu().view(torch.int16).numpy().view(np.uint16)
    vb = v.cpu().view(torch.int16).numpy().view(np.uint16)
    want = O.round_bf16(kv.numpy())
    for b in range(B):
        L = int(lens[b])
        if L < S:
            assert np.array_equal(kb[b, L], want[b, :256]) and np.array_equal(vb[b, L], want[b, 256:])
            kb[b, L] = 0
            vb[b, L] = 0
    assert (kb == 0).all() and (vb == 0).all()


@pytest.mark.parametrize("B,d_model", [(5, 256), (64, 256), (40, 384), (100, 384), (33, 448), (130, 448), (64, 7168), (128, 7168)])
def test_kv_projection_and_record_end_to_end(B, d_model):
    print(f"\n[case] kv append B={B} d_model={d_model}", flush=True)
    g = torch.Generator().manual_seed(410 + B)
    x = torch.randn(B, d_model, generator=g).to(torch.bfloat16)
    w = (torch.randn(d_model, 512, generator=g) * 0.03).to(torch.bfloat16)
    ref = O.linear(O.bits_of(x), O.bits_of(w))                                  # fp64 [B, 512]
    lens = torch.tensor([(11 * b) % 200 for b in range(B)], dtype=torch.int32)
    ctx = U.get_ctx(max_batch=256, max_seq_len=1024, d_model=d_model) if d_model != 7168 else U.get_ctx()
    S = 200
    # bf16 cache
    k = torch.zeros(B, S, 256, dtype=torch.bfloat16).cuda()
    v = torch.zeros(B, S, 256, dtype=torch.bfloat16).cuda()
    mfa.mfa_kv_append(ctx, x.cuda(), w.cuda(), k, v, lens.cuda())
    torch.cuda.synchronize()
    idx = torch.arange(B), lens.long()
    got = torch.cat([k.cpu()[idx], v.cpu()[idx]], dim=1).float().numpy()
    err = U.row_normalised_error(got, ref)
    print(f"   bf16 record vs fp64 projection: row-normalised max error {err:.3e}", flush=True)
    assert err <= TOL_LINEAR
    # fp8 cache: dequantised record against the fp64 projection, within half a code step of the row's scale
    k8 = torch.zeros(B, S, 256, dtype=torch.uint8).cuda().view(torch.float8_e4m3fn)
    v8 = torch.zeros(B, S, 256, dtype=torch.uint8).cuda().view(torch.float8_e4m3fn)
    ks = torch.zeros(B, S).cuda()
    vs = torch.zeros(B, S).cuda()
    mfa.mfa_kv_append(ctx, x.cuda(), w.cuda(), k8, v8, lens.cuda(), ks, vs)
    torch.cuda.synchronize()
    deq = torch.cat([k8.cpu()[idx].float() * ks.cpu()[idx].unsqueeze(1), v8.cpu()[idx].float() * vs.cpu()[idx].unsqueeze(1)],
                    dim=1).numpy()
    amax = np.stack([np.abs(ref[:, :256]).max(1), np.abs(ref[:, 256:]).max(1)], 1).repeat(256, axis=1)
    # e4m3 keeps 4 significant bits: |deq - ref| <= 2^-4 |ref| + half a subnormal step, plus the projection's own error
    bound = 2.0 ** -4 * np.abs(ref) + amax / 448.0 * 2.0 ** -10 + 4e-3 * amax
    assert (np.abs(deq - ref) <= bound).all()
    sc = np.concatenate([ks.cpu()[idx].numpy()[:, None], vs.cpu()[idx].numpy()[:, None]], 1)
    assert np.allclose(sc, amax[:, [0, 256]] / 448.0, rtol=5e-3)


@pytest.mark.parametrize("B,d_model", [(5, 256), (64, 256), (40, 384), (100, 384), (33, 448), (130, 448), (64, 7168), (128, 7168)])
def test_output_projection(B, d_model):
    print(f"\n[case] out proj B={B} d_model={d_model}", flush=True)
    g = torch.Generator().manual_seed(420 + B)
    attn = torch.randn(B, 64, 256, generator=g) * 0.05
    w = (torch.randn(16384, d_model, generator=g) * 0.02).to(torch.bfloat16)
    ctx = U.get_ctx(max_batch=256, max_seq_len=1024, d_model=d_model) if d_model != 7168 else U.get_ctx()
    y = mfa.mfa_out_proj(ctx, attn.cuda(), w.cuda())
    torch.cuda.synchronize()
    ref = O.linear(attn.reshape(B, -1).numpy(), O.bits_of(w))
    err = U.row_normalised_error(y.float().cpu().numpy(), ref)
    print(f"   row-normalised max error {err:.3e}", flush=True)
    assert y.dtype == torch.bfloat16 and tuple(y.shape) == (B, d_model)
    assert err <= TOL_LINEAR


def test_decode_layer_chain_on_a_paged_fp8_cache():
    """query path, append, attention over the lengthened sequences, output projection: one decode step."""
    print("\n[case] decode layer chain", flush=True)
    B = 6
    lens0 = [130, 63, 64, 0, 200, 1]
    pc = W.make_paged_case("layer", 430, [L + 1 for L in lens0], kv_dtype="fp8", spare_pages=4, poison=False)
    qc = W.make_query_proj_case("layerq", 431, B=B)
    g = torch.Generator().manual_seed(432)
    w_kv = (torch.randn(7168, 512, generator=g) * 0.02).to(torch.bfloat16)
    w_o = (torch.randn(16384, 7168, generator=g) * 0.02).to(torch.bfloat16)
    ctx = U.get_ctx()
    kp, vp = pc.k_pool.cuda(), pc.v_pool.cuda()
    ksp, vsp = pc.k_scale_pool.cuda(), pc.v_scale_pool.cuda()
    table = pc.block_table.cuda()
    old = torch.tensor(lens0, dtype=torch.int32).cuda()
    new = torch.tensor([L + 1 for L in lens0], dtype=torch.int32).cuda()
    q = mfa.mfa_query_proj(ctx, qc.x.cuda(), qc.w_qa.cuda(), qc.w_qb.cuda())
    mfa.mfa_kv_append_paged(ctx, qc.x.cuda(), w_kv.cuda(), kp, vp, table, old, ksp, vsp)
    out = mfa.mfa_decode_attn_paged(ctx, q, kp, vp, table, new, 201, ksp, vsp)
    y = mfa.mfa_out_proj(ctx, out, w_o.cuda())
    torch.cuda.synchronize()
    # oracle on the very cache bytes and query bits the GPU produced (staged check of the chain)
    b = O.bits_of
    ref_out = O.decode_attn_paged(b(q.cpu()), b(kp.cpu()), b(vp.cpu()), pc.block_table.numpy(), new.cpu().numpy(), pc.scale,
                                  k_scale_pool=b(ksp.cpu()), v_scale_pool=b(vsp.cpu()), kv_dtype=O.KV_E4M3)
    assert U.row_normalised_error(out.cpu().numpy(), ref_out) <= U.TOL_FP8
    ref_y = O.linear(out.cpu().reshape(B, -1).numpy(), b(w_o))
    assert U.row_normalised_error(y.float().cpu().numpy(), ref_y) <= TOL_LINEAR
    # the appended rows are the record of the projection
    ref_kv = O.linear(b(qc.x), b(w_kv))
    for i, L in enumerate(lens0):
        page, row = int(pc.block_table[i, L // 64]), L % 64
        deq = kp.cpu()[page, row].float().numpy() * float(ksp.cpu()[page, row])
        assert np.abs(deq - ref_kv[i, :256]).max() <= 2.0 ** -4 * np.abs(ref_kv[i, :256]).max() + 1e-6
