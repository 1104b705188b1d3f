"""ctypes front end of the CPU oracle (oracle/mfa_oracle.c).

Test infrastructure only: imported by tests/, by the smoke check and by the
cpu_baseline leg of the benchmark.  Never imported by the GPU library or its
binding.  Arrays are numpy; bf16 travels as uint16 bit patterns and e4m3fn as
uint8 bit patterns so that the oracle sees exactly the bytes the GPU sees.
"""
import ctypes
import os

import numpy as np

from . import build as _build

KV_BF16 = 0
KV_E4M3 = 1
KV_E2M1 = 2      # 4-bit e2m1 elements, two per byte: arrays are [..., D/2] uint8

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.mfa_oracle_decode_bf16.restype = ctypes.c_double
        L.mfa_oracle_decode_bf16.argtypes = [ctypes.c_uint16]
        L.mfa_oracle_decode_e4m3fn.restype = ctypes.c_double
        L.mfa_oracle_decode_e4m3fn.argtypes = [ctypes.c_uint8]
        L.mfa_oracle_decode_e2m1.restype = ctypes.c_double
        L.mfa_oracle_decode_e2m1.argtypes = [ctypes.c_uint8]
        L.mfa_oracle_encode_bf16.restype = ctypes.c_uint16
        L.mfa_oracle_encode_bf16.argtypes = [ctypes.c_double]
        L.mfa_oracle_set_threads.argtypes = [ctypes.c_int]
        L.mfa_oracle_get_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def bits_of(t):
    """torch CPU tensor (bf16 / float8_e4m3fn / float32 / int32) -> numpy view of its bytes."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).numpy()
    return t.numpy()


def set_threads(n):
    lib().mfa_oracle_set_threads(int(n))


def get_threads():
    return int(lib().mfa_oracle_get_threads())


def decode_bf16(bits):
    return float(lib().mfa_oracle_decode_bf16(int(bits)))


def decode_e4m3fn(bits):
    return float(lib().mfa_oracle_decode_e4m3fn(int(bits)))


def decode_e2m1(code):
    return float(lib().mfa_oracle_decode_e2m1(int(code)))


def encode_bf16(x):
    return int(lib().mfa_oracle_encode_bf16(float(x)))


def _rows(rows, B, H):
    if rows is None:
        return B * H, None, None
    rows = np.asarray(rows, dtype=np.int32).reshape(-1, 2)
    rb = np.ascontiguousarray(rows[:, 0])
    rh = np.ascontiguousarray(rows[:, 1])
    return len(rb), rb, rh


def decode_attn(q, k, v, seq_lens, scale, k_scale=None, v_scale=None, kv_dtype=KV_BF16,
                rows=None, return_lse=False):
    """q uint16 [B,H,D]; k,v [B,S,D] uint16 (bf16) or uint8 (e4m3fn), or [B,S,D/2] uint8 (packed e2m1);
    scales fp32 [B,S].

    rows: optional list of (b,h) pairs; then the result is [len(rows), D].
    Returns out fp32 [B,H,D] (or [n_rows,D]) and, if asked, lse float64.
    """
    q = _c(q, np.uint16)
    B, H, D = q.shape
    kd = np.uint16 if kv_dtype == KV_BF16 else np.uint8
    k = _c(k, kd)
    v = _c(v, kd)
    assert k.shape == v.shape and k.shape[0] == B and k.shape[2] == (D // 2 if kv_dtype == KV_E2M1 else D)
    S = k.shape[1]
    k_scale = _c(k_scale, np.float32)
    v_scale = _c(v_scale, np.float32)
    seq_lens = _c(np.asarray(seq_lens, dtype=np.int32), np.int32)
    assert seq_lens.shape == (B,) and int(seq_lens.max(initial=0)) <= S and int(seq_lens.min(initial=0)) >= 0
    n, rb, rh = _rows(rows, B, H)
    out = np.empty((n, D), dtype=np.float32)
    lse = np.empty((n,), dtype=np.float64)
    rc = lib().mfa_oracle_decode_attn(
        _ptr(q), _ptr(k), _ptr(v), _ptr(k_scale), _ptr(v_scale), ctypes.c_int(kv_dtype),
        ctypes.c_int64(S), _ptr(seq_lens), ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(D),
        ctypes.c_double(scale), ctypes.c_int64(n), _ptr(rb), _ptr(rh), _ptr(out), _ptr(lse))
    assert rc == 0, rc
    if rows is None:
        out = out.reshape(B, H, D)
        lse = lse.reshape(B, H)
    return (out, lse) if return_lse else out


def decode_attn_paged(q, k_pool, v_pool, block_table, seq_lens, scale, k_scale_pool=None,
                      v_scale_pool=None, kv_dtype=KV_BF16, rows=None, return_lse=False):
    """k_pool,v_pool [n_pages, page, D]; block_table int32 [B, max_blocks]; scale pools fp32 [n_pages, page]."""
    q = _c(q, np.uint16)
    B, H, D = q.shape
    kd = np.uint16 if kv_dtype == KV_BF16 else np.uint8
    k_pool = _c(k_pool, kd)
    v_pool = _c(v_pool, kd)
    n_pages, page, D2 = k_pool.shape
    assert D2 == (D // 2 if kv_dtype == KV_E2M1 else D) and v_pool.shape == k_pool.shape
    block_table = _c(np.asarray(block_table, dtype=np.int32), np.int32)
    assert block_table.shape[0] == B
    seq_lens = _c(np.asarray(seq_lens, dtype=np.int32), np.int32)
    for b in range(B):
        nb = -(-int(seq_lens[b]) // page)
        assert nb <= block_table.shape[1]
        ids = block_table[b, :nb]
        assert ids.size == 0 or (ids.min() >= 0 and ids.max() < n_pages)
    k_scale_pool = _c(k_scale_pool, np.float32)
    v_scale_pool = _c(v_scale_pool, np.float32)
    n, rb, rh = _rows(rows, B, H)
    out = np.empty((n, D), dtype=np.float32)
    lse = np.empty((n,), dtype=np.float64)
    rc = lib().mfa_oracle_decode_attn_paged(
        _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(k_scale_pool), _ptr(v_scale_pool),
        ctypes.c_int(kv_dtype), ctypes.c_int32(page), _ptr(block_table),
        ctypes.c_int32(block_table.shape[1]), _ptr(seq_lens), ctypes.c_int(B), ctypes.c_int(H),
        ctypes.c_int(D), ctypes.c_double(scale), ctypes.c_int64(n), _ptr(rb), _ptr(rh),
        _ptr(out), _ptr(lse))
    assert rc == 0, rc
    if rows is None:
        out = out.reshape(B, H, D)
        lse = lse.reshape(B, H)
    return (out, lse) if return_lse else out


def attn_weights(q, k, v, seq_lens, scale, b, h, k_scale=None, v_scale=None, kv_dtype=KV_BF16):
    """Normalised attention weights (float64 [L_b]) and output row of one (b,h)."""
    q = _c(q, np.uint16)
    B, H, D = q.shape
    kd = np.uint16 if kv_dtype == KV_BF16 else np.uint8
    k = _c(k, kd)
    v = _c(v, kd)
    S = k.shape[1]
    seq_lens = _c(np.asarray(seq_lens, dtype=np.int32), np.int32)
    w = np.empty((int(seq_lens[b]),), dtype=np.float64)
    row = np.empty((D,), dtype=np.float32)
    rc = lib().mfa_oracle_attn_weights(
        _ptr(q), _ptr(k), _ptr(v), _ptr(_c(k_scale, np.float32)), _ptr(_c(v_scale, np.float32)),
        ctypes.c_int(kv_dtype), ctypes.c_int64(S), _ptr(seq_lens), ctypes.c_int(H), ctypes.c_int(D),
        ctypes.c_double(scale), ctypes.c_int(b), ctypes.c_int(h), _ptr(w), _ptr(row))
    assert rc == 0
    return w, row


def query_proj(x, w_qa, w_qb, eps, gain=None, want_f64=False):
    """x uint16 [B,d_model]; w_qa uint16 [d_model,r]; w_qb uint16 [r,n_out]; gain fp32 [r] or None.

    Returns q as bf16 bit patterns uint16 [B,n_out]; with want_f64 also the
    unrounded float64 query and the normalised low-rank activations.
    """
    x = _c(x, np.uint16)
    w_qa = _c(w_qa, np.uint16)
    w_qb = _c(w_qb, np.uint16)
    gain = _c(gain, np.float32)
    B, d_model = x.shape
    d2, r = w_qa.shape
    r2, n_out = w_qb.shape
    assert d2 == d_model and r2 == r
    q16 = np.empty((B, n_out), dtype=np.uint16)
    q64 = np.empty((B, n_out), dtype=np.float64) if want_f64 else None
    ch = np.empty((B, r), dtype=np.float64) if want_f64 else None
    rc = lib().mfa_oracle_query_proj(
        _ptr(x), _ptr(w_qa), _ptr(gain), _ptr(w_qb), ctypes.c_int(B), ctypes.c_int(d_model),
        ctypes.c_int(r), ctypes.c_int(n_out), ctypes.c_double(eps), _ptr(q16), _ptr(q64), _ptr(ch))
    assert rc == 0, rc
    return (q16, q64, ch) if want_f64 else q16


def linear(a, w):
    """y = a . w in float64.  a: uint16 [B,K] (bf16 bit patterns) or float32 [B,K]; w: uint16 [K,N]."""
    a = np.ascontiguousarray(a)
    assert a.dtype in (np.uint16, np.float32)
    w = _c(w, np.uint16)
    B, K = a.shape
    K2, N = w.shape
    assert K2 == K
    y = np.empty((B, N), dtype=np.float64)
    rc = lib().mfa_oracle_linear(_ptr(a), ctypes.c_int(1 if a.dtype == np.float32 else 0), _ptr(w), ctypes.c_int(B),
                                 ctypes.c_int(K), ctypes.c_int(N), _ptr(y))
    assert rc == 0, rc
    return y


def quantize_rows_e4m3(x):
    """Per-row e4m3fn quantisation in single precision: x float32 [rows, D] -> (codes uint8 [rows, D], scales float32 [rows])."""
    x = _c(x, np.float32)
    rows, D = x.shape
    codes = np.empty((rows, D), dtype=np.uint8)
    scales = np.empty((rows,), dtype=np.float32)
    rc = lib().mfa_oracle_quantize_rows_e4m3(_ptr(x), ctypes.c_int(rows), ctypes.c_int(D), _ptr(codes), _ptr(scales))
    assert rc == 0, rc
    return codes, scales


def quantize_rows_e2m1(x):
    """Per-row e2m1 quantisation in single precision: x float32 [rows, D] -> (packed uint8 [rows, D/2], scales float32 [rows])."""
    x = _c(x, np.float32)
    rows, D = x.shape
    packed = np.empty((rows, D // 2), dtype=np.uint8)
    scales = np.empty((rows,), dtype=np.float32)
    rc = lib().mfa_oracle_quantize_rows_e2m1(_ptr(x), ctypes.c_int(rows), ctypes.c_int(D), _ptr(packed), _ptr(scales))
    assert rc == 0, rc
    return packed, scales


def round_bf16(x):
    """float32 array -> bf16 bit patterns (uint16), nearest with ties to even."""
    x = _c(x, np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    rc = lib().mfa_oracle_round_bf16(_ptr(x), ctypes.c_int64(x.size), _ptr(out))
    assert rc == 0, rc
    return out

