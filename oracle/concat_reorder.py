"""The concat/reorder formulation of dKV-Cache-Decode (Algorithm 1, Appendix A), as a second,
independently organised statement of the same computation (oracle; test infrastructure).

The cache is COMPACT: it holds only the rows of the unmasked positions, in a layout that puts
cached rows on the left and freshly computed rows on the right. Attention runs over that
permuted layout (it has no mask, so the order of keys does not matter), rotary angles follow
each row's true position, and the rows kept for the next step are picked with the index map
of `schedule.reorder_map`. Must agree with the position-indexed store of `sampler.generate`.
"""
import numpy as np
from dkv_inputs.configs import DECODE, CONFIDENCE
from . import schedule as S
from .model import rmsnorm, rope, silu, attention, logits_of
from .sampler import predict, top_k_positions


def generate_decode(model, weights, run, prompt, forced=None):
    """Decode variant, confidence remasking, one sequence at a time. Returns per step
    (candidate positions, candidate logits, committed positions, committed tokens)."""
    assert run.variant == DECODE and run.remask == CONFIDENCE and run.delay == 1
    L, P, k = run.seq_len, run.prompt_len, run.k_per_step
    Hq, Hkv, dh = model.n_q_heads, model.n_kv_heads, model.head_dim
    out = []
    for b in range(run.batch):
        x = np.full(L, model.mask_id, dtype=np.int64)
        x[:P] = prompt[b]
        masked = [p >= P for p in range(L)]
        d_prev = []
        cached_pos = []                               # layout of the compact cache, all layers
        Kc = [np.zeros((Hkv, 0, dh)) for _ in range(model.n_layers)]
        Vc = [np.zeros((Hkv, 0, dh)) for _ in range(model.n_layers)]
        per_step = []
        for t in range(run.steps):
            if S.is_refresh_step(run, t):             # the cached set is emptied
                cached_pos = []
                Kc = [np.zeros((Hkv, 0, dh)) for _ in range(model.n_layers)]
                Vc = [np.zeros((Hkv, 0, dh)) for _ in range(model.n_layers)]
            fresh_pos = [p for p in range(L) if p not in set(cached_pos)]   # M_{t-1}
            assert cached_pos or len(fresh_pos) == L
            if cached_pos:
                assert sorted(fresh_pos) == sorted(set(p for p in range(L) if masked[p]) | set(d_prev))
            layout = cached_pos + fresh_pos                                  # cached left, fresh right
            unmasked_now = [p for p in range(L) if not masked[p]]            # I \ M_t
            _, _, _, take = S.reorder_map(cached_pos, unmasked_now, L)
            h = weights.embed()[x[fresh_pos]].astype(np.float64)
            pe = np.asarray(fresh_pos)                                       # PE' of the right part
            for l in range(model.n_layers):
                w = weights.layer(l)
                a = rmsnorm(h, w["norm1"], model.rms_eps)
                q = rope((a @ w["wq"].T.astype(np.float64)).reshape(-1, Hq, dh), pe, model.rope_theta)
                kf = rope((a @ w["wk"].T.astype(np.float64)).reshape(-1, Hkv, dh), pe, model.rope_theta)
                vf = (a @ w["wv"].T.astype(np.float64)).reshape(-1, Hkv, dh)
                K_all = np.concatenate([Kc[l], np.transpose(kf, (1, 0, 2))], axis=1)   # Concat
                V_all = np.concatenate([Vc[l], np.transpose(vf, (1, 0, 2))], axis=1)
                Kc[l], Vc[l] = K_all[:, take, :], V_all[:, take, :]                    # Reorder
                o = attention(q, K_all, V_all, Hq // Hkv)
                h = h + o.reshape(-1, Hq * dh) @ w["wo"].T.astype(np.float64)
                m = rmsnorm(h, w["norm2"], model.rms_eps)
                h = h + (silu(m @ w["w_gate"].T.astype(np.float64)) * (m @ w["w_up"].T.astype(np.float64))) \
                    @ w["w_down"].T.astype(np.float64)
            cached_pos = list(unmasked_now)
            lo, hi = S.block_range(run, t)
            cand = [p for p in fresh_pos if masked[p] and lo <= p < hi]
            lg = logits_of(model, weights, h[[fresh_pos.index(p) for p in cand]])
            tk, cf = predict(lg, model.mask_id)
            chosen = top_k_positions(cand, cf, k)
            toks = [int(tk[cand.index(p)]) for p in chosen]
            if forced is not None:
                chosen = [int(p) for p in forced[t][0][b]]
                toks = [int(v) for v in forced[t][1][b]]
            for p, v in zip(chosen, toks):
                x[p] = v
                masked[p] = False
            d_prev = chosen
            per_step.append((cand, lg, chosen, toks))
        out.append(per_step)
    return out
