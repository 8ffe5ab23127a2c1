"""8-bit scalar quantisation of the keys for the search (test oracle; see package header).

Appendix C of the paper names scalar quantisation of the KV vectors to 8 bits as the next
step and gives no scheme, so the scheme is this build's reading: per (sequence, KV head)
and per dimension d, symmetric and linear,

    scale_d = max_i |k[i, d]| / 127        (1 when the column is all zero)
    k8[i, d] = clamp(round_half_even(k[i, d] / scale_d), -127, 127)

in float32 arithmetic (each division rounded once), so that a device kernel can produce
the same bytes. Only the graph search reads the quantised keys: it scores
<q * scale, k8>, i.e. the walk is search.greedy_search run on
(scaled_query(q, scale), k8 as float32). Attention (Eq. 1-2)
always uses the original keys and values.
"""
import numpy as np

F32 = np.float32


def quantize_keys(K):
    """K: [N][d] (values exactly representable in float32). Returns (k8 int8 [N][d],
    scale float32 [d])."""
    K = np.asarray(K, F32)
    maxabs = np.abs(K).max(axis=0).astype(F32) if K.shape[0] else np.zeros(K.shape[1], F32)
    scale = (maxabs / F32(127.0)).astype(F32)
    scale[maxabs == 0] = F32(1.0)
    r = np.rint((K / scale[None, :]).astype(F32))          # rint: round half to even
    k8 = np.clip(r, -127, 127).astype(np.int8)
    return k8, scale


def scaled_query(q, scale):
    """q * scale in float32: what the search multiplies the 8-bit keys with."""
    return (np.asarray(q, F32) * np.asarray(scale, F32)).astype(F32)
