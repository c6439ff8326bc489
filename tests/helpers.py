"""Shared test utilities (no method arithmetic of either side)."""
import numpy as np
from dkv_inputs.configs import ModelShape, RunShape, FP32, BF16, DECODE, RANDOM_ORDER, CONFIDENCE
import dkv_inputs as D

SMALL = ModelShape(n_layers=2, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=4, d_ffn=32,
                   vocab=24, mask_id=23, dtype=FP32)


def rel_err(got, ref):
    """(L2 relative error, max-abs error over max-abs reference)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    l2 = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
    mx = np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-300) if ref.size else 0.0
    return l2, mx


def simulate_schedule(run, order=None, seed=0, forced_scopes=None):
    """Drive oracle.schedule alone (no model): commit random candidates (or the fixed order).
    Returns (active[t][b], committed[t][b], stamp history [t] -> array [B, L])."""
    from oracle import schedule as S
    rng = np.random.default_rng(seed)
    B, L, k = run.batch, run.seq_len, run.k_per_step
    masked = np.zeros((B, L), dtype=bool)
    masked[:, run.prompt_len:] = True
    stamp = np.full((B, L), -1, dtype=np.int32)
    d_prev = [[] for _ in range(B)]
    acts, commits, stamps = [], [], []
    for t in range(run.steps):
        a_t, c_t = [], []
        for b in range(B):
            d_cur = None
            if run.remask == RANDOM_ORDER:
                d_cur = [int(p) for p in order[b, t * k:(t + 1) * k]]
            fs = None if forced_scopes is None else forced_scopes.get(t)
            act = S.select_active(run, t, masked[b], d_prev[b], d_cur, fs)
            cand = S.candidates(run, t, act, masked[b])
            chosen = d_cur if d_cur is not None else sorted(rng.choice(cand, size=k, replace=False).tolist())
            stamp[b, act] = t
            a_t.append(act)
            c_t.append(chosen)
        for b in range(B):
            masked[b, c_t[b]] = False
            d_prev[b] = c_t[b]
        acts.append(a_t)
        commits.append(c_t)
        stamps.append(stamp.copy())
    return acts, commits, stamps
