"""Memory-traffic model of one decode-attention step: the paper's element counts (Sec. 3.4,
Eq. 8-10) and the byte counts this build reports bandwidth against.  Pure host arithmetic."""
from __future__ import annotations

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16


def paper_elements_without_relay(b, s, c, d):
    """Eq. 8: queries + cached KVs (system re-read per request) + outputs."""
    return b * d + b * (s + c) * d + b * d


def paper_elements_with_relay(b, s, c, d):
    """Eq. 9: system attention + context attention + relay fusion."""
    return (b * d + s * d + b * d) + (b * d + b * c * d + b * d) + 3 * b * d


def paper_speedup(b, s, c):
    """Eq. 10: p = (s + c + 2) / (s / b + c + 7)."""
    return (s + c + 2.0) / (s / float(b) + c + 7.0)


def ridge_intensity(tflops, gbs):
    """Sec. 3.1: arithmetic intensity above which an operator stops being memory-bound."""
    return tflops * 1e12 / (gbs * 1e9)


def relay_decode_bytes(batch, num_q_heads, num_kv_heads, head_dim, sys_len, total_ctx_tokens,
                       elt=2):
    """Bytes the relay path must move once: q and out, the system K and V once per batch, and
    every request's context K and V once per kv head (K and V counted separately, unlike
    Eq. 9 which counts a key/value pair as one d-vector; fusion traffic is not counted
    because it is not algorithmically required)."""
    qo = 2 * batch * num_q_heads * head_dim * elt
    sys_kv = 2 * sys_len * num_kv_heads * head_dim * elt
    ctx_kv = 2 * total_ctx_tokens * num_kv_heads * head_dim * elt
    return qo + sys_kv + ctx_kv


def naive_decode_bytes(batch, num_q_heads, num_kv_heads, head_dim, sys_len, total_ctx_tokens,
                       elt=2):
    """Per-request attention: the system K and V are read once per request (Eq. 8)."""
    qo = 2 * batch * num_q_heads * head_dim * elt
    kv = 2 * (batch * sys_len + total_ctx_tokens) * num_kv_heads * head_dim * elt
    return qo + kv


def byte_model_speedup(b, s, c):
    """Eq. 10 redone with K and V counted separately and no fusion pass:
    (s + c + 1) / (s / b + c + 1)."""
    return (s + c + 1.0) / (s / float(b) + c + 1.0)
