"""Thin ctypes binding of libmfa.so (the C boundary declared in include/mfa.h).

Argument marshalling only: every step of the decode path runs in the HIP
kernels of the library.  PyTorch supplies device memory (tensors) and the
current HIP stream.  There is no fallback: if the library cannot be loaded the
import of a function from it raises.
"""
import ctypes
import os
from dataclasses import dataclass

import torch

from . import build as _build

MFA_OK = 0
MFA_ERR_INVALID_ARG = 1
MFA_ERR_UNSUPPORTED = 2
MFA_ERR_WORKSPACE_TOO_SMALL = 3
MFA_ERR_HIP = 4
MFA_ERR_HOST_ALLOC = 5

MFA_SCHEDULE_BALANCED = 0
MFA_SCHEDULE_FIXED = 1

MFA_KV_BF16 = 0
MFA_KV_FP8_E4M3 = 1
MFA_KV_FP4_E2M1 = 2

EXPORTS = [
    "mfa_decode_workspace_bytes", "mfa_decode_init", "mfa_decode_destroy", "mfa_status_string",
    "mfa_query_proj", "mfa_decode_attn", "mfa_decode_attn_paged", "mfa_debug_gather_paged",
    "mfa_decode_num_splits", "mfa_debug_set_kernel_events", "mfa_debug_stream_read",
    "mfa_kv_append", "mfa_kv_append_paged", "mfa_debug_kv_record", "mfa_out_proj",
    "mfa_decode_attn_multi", "mfa_decode_attn_paged_multi", "mfa_decode_attn_static",
]


class MfaConfigC(ctypes.Structure):
    _fields_ = [
        ("n_q_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("d_model", ctypes.c_int32),
        ("q_rank", ctypes.c_int32), ("softmax_scale", ctypes.c_float), ("rms_eps", ctypes.c_float),
        ("page_size", ctypes.c_int32), ("max_batch", ctypes.c_int32), ("max_seq_len", ctypes.c_int32),
        ("device", ctypes.c_int32), ("target_workgroups", ctypes.c_int32), ("schedule", ctypes.c_int32),
    ]


@dataclass
class MfaConfig:
    n_q_heads: int = 64
    head_dim: int = 256
    d_model: int = 7168
    q_rank: int = 2048
    softmax_scale: float = 1.0 / 16.0
    rms_eps: float = 1e-6
    page_size: int = 64
    max_batch: int = 128
    max_seq_len: int = 32768
    device: int = 0
    target_workgroups: int = 0          # 0: the library's default (one per compute unit)
    schedule: int = MFA_SCHEDULE_BALANCED

    def to_c(self):
        return MfaConfigC(self.n_q_heads, self.head_dim, self.d_model, self.q_rank, self.softmax_scale,
                          self.rms_eps, self.page_size, self.max_batch, self.max_seq_len, self.device,
                          self.target_workgroups, self.schedule)


_lib = None


def lib_path():
    return _build.LIB


def lib():
    """Load libmfa.so (building it first only if no built library exists; a library older than its sources
    is loaded as it is, with a warning: rebuild with `python -m paper_2507_19427_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        _build.build(force=True)
    elif path == _build.LIB and _build._stale():
        import warnings
        warnings.warn(f"{path} is older than the sources under csrc/: the tests and benchmarks run the OLD binary "
                      "until it is rebuilt (python -m paper_2507_19427_amd.build)", RuntimeWarning, stacklevel=2)
    L = ctypes.CDLL(path)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    cfgp = ctypes.POINTER(MfaConfigC)
    L.mfa_decode_workspace_bytes.restype = sz
    L.mfa_decode_workspace_bytes.argtypes = [cfgp]
    L.mfa_decode_init.restype = ctypes.c_int
    L.mfa_decode_init.argtypes = [cfgp, vp, sz, ctypes.POINTER(vp)]
    L.mfa_decode_destroy.restype = None
    L.mfa_decode_destroy.argtypes = [vp]
    L.mfa_status_string.restype = ctypes.c_char_p
    L.mfa_status_string.argtypes = [ctypes.c_int]
    L.mfa_query_proj.restype = ctypes.c_int
    L.mfa_query_proj.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp]
    L.mfa_decode_attn.restype = ctypes.c_int
    L.mfa_decode_attn.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int, i64, vp, i32, i32, vp, vp]
    L.mfa_decode_attn_static.restype = ctypes.c_int
    L.mfa_decode_attn_static.argtypes = L.mfa_decode_attn.argtypes
    L.mfa_decode_attn_paged.restype = ctypes.c_int
    L.mfa_decode_attn_paged.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int, i32, vp, i32, vp, i32, i32, vp, vp]
    L.mfa_decode_attn_multi.restype = ctypes.c_int
    L.mfa_decode_attn_multi.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int, i64, vp, i32, i32, i32, vp, vp]
    L.mfa_decode_attn_paged_multi.restype = ctypes.c_int
    L.mfa_decode_attn_paged_multi.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int, i32, vp, i32, vp, i32, i32, i32,
                                              vp, vp]
    L.mfa_debug_gather_paged.restype = ctypes.c_int
    L.mfa_debug_gather_paged.argtypes = [vp, vp, i32, i32, vp, i32, vp, i32, i32, vp, i64, vp]
    L.mfa_debug_set_kernel_events.restype = ctypes.c_int
    L.mfa_debug_set_kernel_events.argtypes = [vp, vp, vp]
    L.mfa_debug_stream_read.restype = ctypes.c_int
    L.mfa_debug_stream_read.argtypes = [vp, vp, vp, sz, vp]
    L.mfa_decode_num_splits.restype = i32
    L.mfa_decode_num_splits.argtypes = [vp, i32, i32]
    L.mfa_kv_append.restype = ctypes.c_int
    L.mfa_kv_append.argtypes = [vp, vp, vp, ctypes.c_int, vp, vp, vp, vp, i64, vp, i32, vp]
    L.mfa_kv_append_paged.restype = ctypes.c_int
    L.mfa_kv_append_paged.argtypes = [vp, vp, vp, ctypes.c_int, vp, vp, vp, vp, i32, vp, i32, vp, i32, vp]
    L.mfa_debug_kv_record.restype = ctypes.c_int
    L.mfa_debug_kv_record.argtypes = [vp, vp, ctypes.c_int, vp, vp, vp, vp, i64, vp, i32, vp, i32, vp]
    L.mfa_out_proj.restype = ctypes.c_int
    L.mfa_out_proj.argtypes = [vp, vp, vp, vp, i32, vp]
    _lib = L
    return L


class MfaError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().mfa_status_string(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


def _check(status, where):
    if status != MFA_OK:
        raise MfaError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _kv_dtype(t):
    if t.dtype == torch.bfloat16:
        return MFA_KV_BF16
    if t.dtype == torch.float8_e4m3fn:
        return MFA_KV_FP8_E4M3
    if t.dtype == torch.uint8:                       # e2m1 codes, two per byte: last dimension head_dim / 2
        return MFA_KV_FP4_E2M1
    raise TypeError(f"unsupported cache dtype {t.dtype}")


def _cache_width(cfg, kvd):
    """Last dimension of a cache tensor: elements per row, or bytes for the packed 4-bit record."""
    return cfg.head_dim // 2 if kvd == MFA_KV_FP4_E2M1 else cfg.head_dim


def _want(t, dtype, name):
    if t.dtype != dtype or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name}: expected contiguous device tensor of {dtype}, got {t.dtype} on {t.device}")


def mfa_decode_workspace_bytes(cfg: MfaConfig) -> int:
    c = cfg.to_c()
    return int(lib().mfa_decode_workspace_bytes(ctypes.byref(c)))


class MfaContext:
    """Owns the device workspace (a torch tensor) and the library context handle."""

    def __init__(self, cfg: MfaConfig):
        self.cfg = cfg
        nbytes = mfa_decode_workspace_bytes(cfg)
        if nbytes == 0:
            raise MfaError(MFA_ERR_UNSUPPORTED, "mfa_decode_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=f"cuda:{cfg.device}")
        handle = ctypes.c_void_p()
        c = cfg.to_c()
        with torch.cuda.device(cfg.device):
            _check(lib().mfa_decode_init(ctypes.byref(c), _ptr(self.workspace), nbytes, ctypes.byref(handle)),
                   "mfa_decode_init")
        self.handle = handle

    def close(self):
        if getattr(self, "handle", None):
            lib().mfa_decode_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def mfa_decode_init(cfg: MfaConfig) -> MfaContext:
    return MfaContext(cfg)


def mfa_decode_num_splits(ctx: MfaContext, B: int, max_seq_len_hint: int) -> int:
    return int(lib().mfa_decode_num_splits(ctx.handle, B, max_seq_len_hint))


def mfa_query_proj(ctx: MfaContext, x, w_qa, w_qb, rms_gain=None, q_out=None):
    """x bf16 [B,d_model], w_qa bf16 [d_model,r], w_qb bf16 [r,H*D] -> q bf16 [B,H,D]."""
    cfg = ctx.cfg
    for t, nm in ((x, "x"), (w_qa, "w_qa"), (w_qb, "w_qb")):
        _want(t, torch.bfloat16, nm)
    B = x.shape[0]
    if tuple(x.shape) != (B, cfg.d_model) or tuple(w_qa.shape) != (cfg.d_model, cfg.q_rank) or \
            tuple(w_qb.shape) != (cfg.q_rank, cfg.n_q_heads * cfg.head_dim):
        raise ValueError("query path shapes do not match the context configuration")
    if rms_gain is not None:
        _want(rms_gain, torch.float32, "rms_gain")
        if tuple(rms_gain.shape) != (cfg.q_rank,):
            raise ValueError("rms_gain shape")
    if q_out is None:
        q_out = torch.empty(B, cfg.n_q_heads, cfg.head_dim, dtype=torch.bfloat16, device=x.device)
    else:
        _want(q_out, torch.bfloat16, "q_out")
    _check(lib().mfa_query_proj(ctx.handle, _ptr(x), _ptr(w_qa), _ptr(rms_gain), _ptr(w_qb), _ptr(q_out), B,
                                _stream()), "mfa_query_proj")
    return q_out


def mfa_decode_attn(ctx: MfaContext, q, k_cache, v_cache, seq_lens, max_seq_len_hint, k_scale=None,
                    v_scale=None, out=None, _entry="mfa_decode_attn"):
    """q bf16 [B,H,D]; k_cache,v_cache [B,S,D] bf16 or float8_e4m3fn; seq_lens int32 [B] on device."""
    cfg = ctx.cfg
    _want(q, torch.bfloat16, "q")
    _want(seq_lens, torch.int32, "seq_lens")
    B = q.shape[0]
    kvd = _kv_dtype(k_cache)
    if v_cache.dtype != k_cache.dtype or not k_cache.is_contiguous() or not v_cache.is_contiguous():
        raise TypeError("k_cache / v_cache must be contiguous and of one dtype")
    S = k_cache.shape[1]
    width = _cache_width(cfg, kvd)
    if tuple(q.shape) != (B, cfg.n_q_heads, cfg.head_dim) or tuple(k_cache.shape) != (B, S, width) or \
            tuple(v_cache.shape) != (B, S, width) or tuple(seq_lens.shape) != (B,):
        raise ValueError("attention shapes do not match")
    for t, nm in ((k_scale, "k_scale"), (v_scale, "v_scale")):
        if t is not None:
            _want(t, torch.float32, nm)
            if tuple(t.shape) != (B, S):
                raise ValueError(nm + " shape")
    if out is None:
        out = torch.empty(B, cfg.n_q_heads, cfg.head_dim, dtype=torch.float32, device=q.device)
    else:
        _want(out, torch.float32, "out")
        if tuple(out.shape) != (B, cfg.n_q_heads, cfg.head_dim):
            raise ValueError("out shape")
    _check(getattr(lib(), _entry)(ctx.handle, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale),
                                  kvd, S, _ptr(seq_lens), int(max_seq_len_hint), B, _ptr(out), _stream()), _entry)
    return out


def mfa_decode_attn_static(ctx: MfaContext, q, k_cache, v_cache, seq_lens, max_seq_len_hint, out, k_scale=None,
                           v_scale=None):
    """mfa_decode_attn with the partial results in the library's fixed device array instead of the context's
    workspace (for callers that cannot allocate); `out` is the caller's, nothing is allocated here either."""
    if out is None:
        raise ValueError("mfa_decode_attn_static writes into the caller's `out`")
    return mfa_decode_attn(ctx, q, k_cache, v_cache, seq_lens, max_seq_len_hint, k_scale=k_scale, v_scale=v_scale,
                           out=out, _entry="mfa_decode_attn_static")


def mfa_decode_attn_paged(ctx: MfaContext, q, k_pool, v_pool, block_table, seq_lens, max_seq_len_hint,
                          k_scale_pool=None, v_scale_pool=None, out=None):
    """k_pool,v_pool [n_pages,page,D]; block_table int32 [B,max_blocks] on device."""
    cfg = ctx.cfg
    _want(q, torch.bfloat16, "q")
    _want(seq_lens, torch.int32, "seq_lens")
    _want(block_table, torch.int32, "block_table")
    B = q.shape[0]
    kvd = _kv_dtype(k_pool)
    if v_pool.dtype != k_pool.dtype or not k_pool.is_contiguous() or not v_pool.is_contiguous():
        raise TypeError("k_pool / v_pool must be contiguous and of one dtype")
    n_pages = k_pool.shape[0]
    if tuple(k_pool.shape) != (n_pages, cfg.page_size, _cache_width(cfg, kvd)) or tuple(v_pool.shape) != tuple(k_pool.shape) \
            or block_table.shape[0] != B or tuple(seq_lens.shape) != (B,) or \
            tuple(q.shape) != (B, cfg.n_q_heads, cfg.head_dim):
        raise ValueError("paged attention shapes do not match")
    for t, nm in ((k_scale_pool, "k_scale_pool"), (v_scale_pool, "v_scale_pool")):
        if t is not None:
            _want(t, torch.float32, nm)
            if tuple(t.shape) != (n_pages, cfg.page_size):
                raise ValueError(nm + " shape")
    if out is None:
        out = torch.empty(B, cfg.n_q_heads, cfg.head_dim, dtype=torch.float32, device=q.device)
    else:
        _want(out, torch.float32, "out")
        if tuple(out.shape) != (B, cfg.n_q_heads, cfg.head_dim):
            raise ValueError("out shape")
    _check(lib().mfa_decode_attn_paged(ctx.handle, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(k_scale_pool),
                                       _ptr(v_scale_pool), kvd, n_pages, _ptr(block_table), block_table.shape[1],
                                       _ptr(seq_lens), int(max_seq_len_hint), B, _ptr(out), _stream()),
           "mfa_decode_attn_paged")
    return out


def mfa_decode_attn_multi(ctx: MfaContext, q, k_cache, v_cache, seq_lens, max_seq_len_hint, k_scale=None,
                          v_scale=None, out=None):
    """q bf16 [B,q_len,H,D]; caches as for mfa_decode_attn; out fp32 [B,q_len,H,D]."""
    cfg = ctx.cfg
    _want(q, torch.bfloat16, "q")
    _want(seq_lens, torch.int32, "seq_lens")
    if q.dim() != 4:
        raise ValueError("q must be [B, q_len, H, D]")
    B, q_len = q.shape[0], q.shape[1]
    kvd = _kv_dtype(k_cache)
    if v_cache.dtype != k_cache.dtype or not k_cache.is_contiguous() or not v_cache.is_contiguous():
        raise TypeError("k_cache / v_cache must be contiguous and of one dtype")
    S = k_cache.shape[1]
    width = _cache_width(cfg, kvd)
    if tuple(q.shape) != (B, q_len, cfg.n_q_heads, cfg.head_dim) or tuple(k_cache.shape) != (B, S, width) or \
            tuple(v_cache.shape) != (B, S, width) or tuple(seq_lens.shape) != (B,):
        raise ValueError("attention shapes do not match")
    for t, nm in ((k_scale, "k_scale"), (v_scale, "v_scale")):
        if t is not None:
            _want(t, torch.float32, nm)
            if tuple(t.shape) != (B, S):
                raise ValueError(nm + " shape")
    if out is None:
        out = torch.empty(B, q_len, cfg.n_q_heads, cfg.head_dim, dtype=torch.float32, device=q.device)
    else:
        _want(out, torch.float32, "out")
        if tuple(out.shape) != tuple(q.shape):
            raise ValueError("out shape")
    _check(lib().mfa_decode_attn_multi(ctx.handle, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale),
                                       _ptr(v_scale), kvd, S, _ptr(seq_lens), int(max_seq_len_hint), B, q_len,
                                       _ptr(out), _stream()), "mfa_decode_attn_multi")
    return out


def mfa_decode_attn_paged_multi(ctx: MfaContext, q, k_pool, v_pool, block_table, seq_lens, max_seq_len_hint,
                                k_scale_pool=None, v_scale_pool=None, out=None):
    """q bf16 [B,q_len,H,D]; pools and table as for mfa_decode_attn_paged; out fp32 [B,q_len,H,D]."""
    cfg = ctx.cfg
    _want(q, torch.bfloat16, "q")
    _want(seq_lens, torch.int32, "seq_lens")
    _want(block_table, torch.int32, "block_table")
    if q.dim() != 4:
        raise ValueError("q must be [B, q_len, H, D]")
    B, q_len = q.shape[0], q.shape[1]
    kvd = _kv_dtype(k_pool)
    if v_pool.dtype != k_pool.dtype or not k_pool.is_contiguous() or not v_pool.is_contiguous():
        raise TypeError("k_pool / v_pool must be contiguous and of one dtype")
    n_pages = k_pool.shape[0]
    if tuple(k_pool.shape) != (n_pages, cfg.page_size, _cache_width(cfg, kvd)) or tuple(v_pool.shape) != tuple(k_pool.shape) \
            or block_table.shape[0] != B or tuple(seq_lens.shape) != (B,) or \
            tuple(q.shape) != (B, q_len, cfg.n_q_heads, cfg.head_dim):
        raise ValueError("paged attention shapes do not match")
    for t, nm in ((k_scale_pool, "k_scale_pool"), (v_scale_pool, "v_scale_pool")):
        if t is not None:
            _want(t, torch.float32, nm)
            if tuple(t.shape) != (n_pages, cfg.page_size):
                raise ValueError(nm + " shape")
    if out is None:
        out = torch.empty(B, q_len, cfg.n_q_heads, cfg.head_dim, dtype=torch.float32, device=q.device)
    else:
        _want(out, torch.float32, "out")
        if tuple(out.shape) != tuple(q.shape):
            raise ValueError("out shape")
    _check(lib().mfa_decode_attn_paged_multi(ctx.handle, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(k_scale_pool),
                                             _ptr(v_scale_pool), kvd, n_pages, _ptr(block_table),
                                             block_table.shape[1], _ptr(seq_lens), int(max_seq_len_hint), B, q_len,
                                             _ptr(out), _stream()), "mfa_decode_attn_paged_multi")
    return out


def mfa_debug_gather_paged(ctx: MfaContext, pool, block_table, seq_lens, max_seq_len_hint, dst):
    """Copy rows j < seq_lens[b] of every sequence from pool [n_pages,page,...] into dst [B,S,...]."""
    row_bytes = pool[0, 0].numel() * pool.element_size()
    B = block_table.shape[0]
    _check(lib().mfa_debug_gather_paged(ctx.handle, _ptr(pool), row_bytes, pool.shape[0], _ptr(block_table),
                                        block_table.shape[1], _ptr(seq_lens), int(max_seq_len_hint), B, _ptr(dst),
                                        dst.shape[1], _stream()), "mfa_debug_gather_paged")
    return dst


def mfa_debug_set_kernel_events(ctx: MfaContext, ev_before=None, ev_after=None):
    """Record the two torch.cuda.Event objects (timing enabled, already recorded once so that their
    HIP handles exist) around the streaming kernel of every later attention call; None, None stops."""
    hb = None if ev_before is None else ctypes.c_void_p(ev_before.cuda_event)
    ha = None if ev_after is None else ctypes.c_void_p(ev_after.cuda_event)
    _check(lib().mfa_debug_set_kernel_events(ctx.handle, hb, ha), "mfa_debug_set_kernel_events")


def mfa_debug_stream_read(ctx: MfaContext, a, b):
    """Read the two equally sized device tensors once with a do-nothing kernel (bandwidth ceiling probe)."""
    nbytes = a.numel() * a.element_size()
    if b.numel() * b.element_size() != nbytes:
        raise ValueError("buffers must have equal size")
    _check(lib().mfa_debug_stream_read(ctx.handle, _ptr(a), _ptr(b), nbytes, _stream()), "mfa_debug_stream_read")


def _check_cache_pair(k, v, ks, vs, rows_shape):
    kvd = _kv_dtype(k)
    if v.dtype != k.dtype or not k.is_contiguous() or not v.is_contiguous() or tuple(v.shape) != tuple(k.shape):
        raise TypeError("key and value caches must be contiguous, of one dtype and one shape")
    for t, nm in ((ks, "k_scale"), (vs, "v_scale")):
        if t is not None:
            _want(t, torch.float32, nm)
            if tuple(t.shape) != tuple(rows_shape):
                raise ValueError(nm + " shape")
    return kvd


def mfa_kv_append(ctx: MfaContext, x, w_kv, k_cache, v_cache, seq_lens, k_scale=None, v_scale=None):
    """x bf16 [B,d_model], w_kv bf16 [d_model, 2*head_dim]; writes row seq_lens[b] of k_cache/v_cache [B,S,D]."""
    cfg = ctx.cfg
    _want(x, torch.bfloat16, "x")
    _want(w_kv, torch.bfloat16, "w_kv")
    _want(seq_lens, torch.int32, "seq_lens")
    B = x.shape[0]
    if tuple(x.shape) != (B, cfg.d_model) or tuple(w_kv.shape) != (cfg.d_model, 2 * cfg.head_dim) or \
            k_cache.dim() != 3 or k_cache.shape[0] != B or k_cache.shape[2] != _cache_width(cfg, _kv_dtype(k_cache)) or \
            tuple(seq_lens.shape) != (B,):
        raise ValueError("kv append shapes do not match")
    kvd = _check_cache_pair(k_cache, v_cache, k_scale, v_scale, k_cache.shape[:2])
    _check(lib().mfa_kv_append(ctx.handle, _ptr(x), _ptr(w_kv), kvd, _ptr(k_cache), _ptr(v_cache), _ptr(k_scale),
                               _ptr(v_scale), k_cache.shape[1], _ptr(seq_lens), B, _stream()), "mfa_kv_append")


def mfa_kv_append_paged(ctx: MfaContext, x, w_kv, k_pool, v_pool, block_table, seq_lens, k_scale_pool=None,
                        v_scale_pool=None):
    """The same into pools [n_pages,page,D] behind block_table int32 [B,max_blocks]."""
    cfg = ctx.cfg
    _want(x, torch.bfloat16, "x")
    _want(w_kv, torch.bfloat16, "w_kv")
    _want(seq_lens, torch.int32, "seq_lens")
    _want(block_table, torch.int32, "block_table")
    B = x.shape[0]
    n_pages = k_pool.shape[0]
    if tuple(x.shape) != (B, cfg.d_model) or tuple(w_kv.shape) != (cfg.d_model, 2 * cfg.head_dim) or \
            tuple(k_pool.shape) != (n_pages, cfg.page_size, _cache_width(cfg, _kv_dtype(k_pool))) or \
            block_table.shape[0] != B or tuple(seq_lens.shape) != (B,):
        raise ValueError("paged kv append shapes do not match")
    kvd = _check_cache_pair(k_pool, v_pool, k_scale_pool, v_scale_pool, k_pool.shape[:2])
    _check(lib().mfa_kv_append_paged(ctx.handle, _ptr(x), _ptr(w_kv), kvd, _ptr(k_pool), _ptr(v_pool), _ptr(k_scale_pool),
                                     _ptr(v_scale_pool), n_pages, _ptr(block_table), block_table.shape[1], _ptr(seq_lens),
                                     B, _stream()), "mfa_kv_append_paged")


def mfa_debug_kv_record(ctx: MfaContext, kv, k_cache, v_cache, seq_lens, k_scale=None, v_scale=None, block_table=None):
    """Write given fp32 rows kv [B, 2*head_dim] as the new token's record (contiguous [B,S,D] or pools + block_table)."""
    _want(kv, torch.float32, "kv")
    _want(seq_lens, torch.int32, "seq_lens")
    B = kv.shape[0]
    kvd = _check_cache_pair(k_cache, v_cache, k_scale, v_scale, k_cache.shape[:2])
    stride = 0 if block_table is not None else k_cache.shape[1]
    width = block_table.shape[1] if block_table is not None else 0
    _check(lib().mfa_debug_kv_record(ctx.handle, _ptr(kv), kvd, _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale),
                                     stride, _ptr(block_table), width, _ptr(seq_lens), B, _stream()), "mfa_debug_kv_record")


def mfa_out_proj(ctx: MfaContext, attn_out, w_o, y=None):
    """attn_out fp32 [B,H,D] (or [B,H*D]), w_o bf16 [H*D, d_model] -> y bf16 [B, d_model]."""
    cfg = ctx.cfg
    _want(attn_out, torch.float32, "attn_out")
    _want(w_o, torch.bfloat16, "w_o")
    B = attn_out.shape[0]
    n_in = cfg.n_q_heads * cfg.head_dim
    if attn_out.numel() != B * n_in or tuple(w_o.shape) != (n_in, cfg.d_model):
        raise ValueError("output projection shapes do not match")
    if y is None:
        y = torch.empty(B, cfg.d_model, dtype=torch.bfloat16, device=attn_out.device)
    else:
        _want(y, torch.bfloat16, "y")
    _check(lib().mfa_out_proj(ctx.handle, _ptr(attn_out), _ptr(w_o), _ptr(y), B, _stream()), "mfa_out_proj")
    return y


class PreparedDecodeAttn:
    """mfa_decode_attn (q [B,H,D]) or mfa_decode_attn_multi (q [B,q_len,H,D]) with its arguments marshalled
    once: calling the object only crosses the C boundary (for loops that must not pay Python-side checks
    per step).  The tensors are kept alive.  The work is enqueued on the stream that is current when the
    object is called (not the one that was current when it was made)."""

    def __init__(self, ctx: MfaContext, q, k_cache, v_cache, seq_lens, max_seq_len_hint, out, k_scale=None,
                 v_scale=None):
        multi = q.dim() == 4
        check = mfa_decode_attn_multi if multi else mfa_decode_attn
        check(ctx, q, k_cache, v_cache, seq_lens, max_seq_len_hint, k_scale=k_scale, v_scale=v_scale,
              out=out)                                 # validates shapes and types once
        self._keep = (ctx, q, k_cache, v_cache, seq_lens, out, k_scale, v_scale)
        self._name = "mfa_decode_attn_multi" if multi else "mfa_decode_attn"
        self._fn = getattr(lib(), self._name)
        head = (ctx.handle, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_scale), _ptr(v_scale),
                _kv_dtype(k_cache), k_cache.shape[1], _ptr(seq_lens), int(max_seq_len_hint), q.shape[0])
        self._args = head + ((q.shape[1],) if multi else ()) + (_ptr(out),)

    def __call__(self):
        st = self._fn(*self._args, _stream())
        if st != MFA_OK:
            raise MfaError(st, self._name)
