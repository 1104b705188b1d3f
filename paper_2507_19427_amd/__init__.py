"""MI355X-native decode-step Multi-Matrix Factorization Attention (MFA).

The product is libmfa.so (HIP kernels behind the C boundary of include/mfa.h);
this package is its thin Python binding plus the seeded workload generators.
"""
from .binding import (  # noqa: F401
    MFA_OK, MFA_ERR_INVALID_ARG, MFA_ERR_UNSUPPORTED, MFA_ERR_WORKSPACE_TOO_SMALL, MFA_ERR_HIP, MFA_ERR_HOST_ALLOC,
    MFA_SCHEDULE_BALANCED, MFA_SCHEDULE_FIXED,
    MFA_KV_BF16, MFA_KV_FP8_E4M3, MFA_KV_FP4_E2M1, MfaConfig, MfaContext, MfaError,
    mfa_decode_workspace_bytes, mfa_decode_init, mfa_decode_num_splits, mfa_query_proj,
    mfa_decode_attn, mfa_decode_attn_paged, mfa_debug_gather_paged, mfa_debug_set_kernel_events, mfa_debug_stream_read,
    mfa_kv_append, mfa_kv_append_paged, mfa_debug_kv_record, mfa_out_proj,
    mfa_decode_attn_multi, mfa_decode_attn_paged_multi, mfa_decode_attn_static,
    PreparedDecodeAttn,
)
