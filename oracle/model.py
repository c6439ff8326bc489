"""Partial transformer forward over a position-indexed K/V store (oracle; test infrastructure).

Everything is float64 numpy. The block is the pre-norm decoder block the benchmark
configurations describe (RMSNorm, rotary embedding, bidirectional attention with optional
grouped K/V heads, SwiGLU), without biases and without any attention mask. Only the rows of
the active set are pushed through; every other position contributes the K/V stored for it
at an earlier step (Eq. 4; Algorithm 1 lines 3-6).
"""
import numpy as np


def rmsnorm(h, gain, eps):
    """Row-wise h / sqrt(mean(h^2) + eps) * gain."""
    h = np.asarray(h, dtype=np.float64)
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h / np.sqrt(ms + eps) * np.asarray(gain, dtype=np.float64)


def rope(x, pos, theta):
    """Rotary embedding, half-split pairing: element i is rotated together with i + dh/2 by the
    angle pos * theta^(-2i/dh). x is [n, heads, dh], pos is [n]. The rotation follows the true
    sequence position of each row, wherever the row sits in the compacted batch (Appendix A)."""
    x = np.asarray(x, dtype=np.float64)
    dh = x.shape[-1]
    half = dh // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax(s, axis=-1):
    m = np.max(s, axis=axis, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=axis, keepdims=True)


def attention(q, K, V, group):
    """Bidirectional attention of n query rows over ALL stored positions.

    q [n, Hq, dh]; K, V [Hkv, L, dh]; query head h reads K/V head h // group.
    Returns [n, Hq, dh]. No mask: every query sees every position (Eq. 4)."""
    n, Hq, dh = q.shape
    out = np.empty_like(q)
    for h in range(Hq):
        kv = h // group
        scores = q[:, h, :] @ K[kv].T / np.sqrt(dh)
        out[:, h, :] = softmax(scores, axis=-1) @ V[kv]
    return out


class KVStore:
    """K and V of every layer, indexed by sequence position: [layer][batch][kv_head][L][dh].
    Rows never written hold NaN, so reading one poisons the result. stamp[b][p] is the last
    step that wrote position p (-1 = never)."""

    def __init__(self, model, batch, seq_len):
        shape = (model.n_layers, batch, model.n_kv_heads, seq_len, model.head_dim)
        self.K = np.full(shape, np.nan, dtype=np.float64)
        self.V = np.full(shape, np.nan, dtype=np.float64)
        self.stamp = np.full((batch, seq_len), -1, dtype=np.int32)


def layer_forward(model, w, h, pos, off, K_l, V_l):
    """One pre-norm block on the active rows (Algorithm 1 lines 3-6 for one layer).

    h [R, d] residual stream entering the layer, rows ordered sequence by sequence; pos [R] their
    sequence positions; off [B+1] row offsets of the sequences; w the layer's weights;
    K_l, V_l [B][Hkv][L][dh] the layer's position-indexed store, whose rows at the active
    positions are overwritten with the fresh post-rotation K and V before attending (Eq. 4).
    Returns the residual stream leaving the layer."""
    Hq, Hkv, dh = model.n_q_heads, model.n_kv_heads, model.head_dim
    group = Hq // Hkv
    B = len(off) - 1
    a = rmsnorm(h, w["norm1"], model.rms_eps)
    q = (a @ np.asarray(w["wq"], dtype=np.float64).T).reshape(-1, Hq, dh)
    k = (a @ np.asarray(w["wk"], dtype=np.float64).T).reshape(-1, Hkv, dh)
    v = (a @ np.asarray(w["wv"], dtype=np.float64).T).reshape(-1, Hkv, dh)
    q = rope(q, pos, model.rope_theta)
    k = rope(k, pos, model.rope_theta)
    o = np.empty_like(q)
    for b in range(B):
        r = slice(off[b], off[b + 1])
        p = pos[r]
        K_l[b][:, p, :] = np.transpose(k[r], (1, 0, 2))
        V_l[b][:, p, :] = np.transpose(v[r], (1, 0, 2))
        o[r] = attention(q[r], K_l[b], V_l[b], group)
    h = h + o.reshape(-1, Hq * dh) @ np.asarray(w["wo"], dtype=np.float64).T
    m = rmsnorm(h, w["norm2"], model.rms_eps)
    gate = m @ np.asarray(w["w_gate"], dtype=np.float64).T
    up = m @ np.asarray(w["w_up"], dtype=np.float64).T
    return h + (silu(gate) * up) @ np.asarray(w["w_down"], dtype=np.float64).T


def forward_active(model, weights, tokens, active, store, t, keep_hidden=None):
    """One model call on the active rows.

    tokens [B, L] current ids; active: list over sequences of sorted position lists.
    Writes the fresh (post-rotation) K and V of the active rows into `store`, stamps them with
    t, and returns the final hidden states h [R, d] (before the final norm), rows ordered
    sequence by sequence, position ascending. `keep_hidden`, if a list, receives the
    residual stream after every layer.
    """
    B = len(active)
    counts = [len(a) for a in active]
    off = np.concatenate([[0], np.cumsum(counts)]).astype(int)
    pos = np.concatenate([np.asarray(a, dtype=np.int64) for a in active]) if off[-1] else np.zeros(0, np.int64)
    seq = np.concatenate([np.full(c, b, dtype=np.int64) for b, c in enumerate(counts)]) if off[-1] else np.zeros(0, np.int64)
    embed = weights.embed()
    h = embed[tokens[seq, pos]].astype(np.float64)
    for l in range(model.n_layers):
        h = layer_forward(model, weights.layer(l), h, pos, off, store.K[l], store.V[l])
        if keep_hidden is not None:
            keep_hidden.append(h.copy())
    for b in range(B):
        store.stamp[b, pos[off[b]:off[b + 1]]] = t
    return h


def logits_of(model, weights, h_rows):
    """Final norm and vocabulary projection of the given hidden rows: [n, V] float64."""
    a = rmsnorm(h_rows, weights.final_norm(), model.rms_eps)
    return a @ np.asarray(weights.lm_head(), dtype=np.float64).T


def full_forward(model, weights, tokens):
    """Cache-free reference: every position recomputed. Returns (h [B*L, d], store)."""
    B, L = tokens.shape
    store = KVStore(model, B, L)
    h = forward_active(model, weights, tokens, [list(range(L))] * B, store, 0)
    return h, store
