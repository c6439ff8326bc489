"""Scatter-then-attend on a position-indexed K/V cache, in isolation (oracle; test infrastructure).

The fresh K/V rows of the active positions replace the stored rows (Algorithm 1 line 4 in a
position-indexed layout), then every active query attends, unmasked, over all L positions
(Eq. 4). float64 throughout.
"""
import numpy as np
from .model import attention


def attn_update(k_cache, v_cache, q, k_new, v_new, active_idx, active_off):
    """k_cache, v_cache [B, Hkv, L, dh] (updated in place, float64); q [R, Hq, dh];
    k_new, v_new [R, Hkv, dh]; active_idx [R]; active_off [B+1]. Returns out [R, Hq, dh]."""
    B = k_cache.shape[0]
    Hq, Hkv = q.shape[1], k_cache.shape[1]
    out = np.empty(q.shape, dtype=np.float64)
    for b in range(B):
        r = slice(int(active_off[b]), int(active_off[b + 1]))
        p = np.asarray(active_idx[r], dtype=np.int64)
        k_cache[b][:, p, :] = np.transpose(k_new[r], (1, 0, 2))
        v_cache[b][:, p, :] = np.transpose(v_new[r], (1, 0, 2))
        out[r] = attention(np.asarray(q[r], dtype=np.float64), k_cache[b], v_cache[b], Hq // Hkv)
    return out
