"""Literal, scalar-loop reconstruction of Eq. 4 from the full K/V history, for tiny cases only
(oracle; test infrastructure).

Nothing is overwritten: the K and V rows computed at every step are kept, and the full
matrices K_t^I, V_t^I of step t are assembled position by position as "the row computed at the
last step s <= t at which this position was among the recomputed rows". The transformer
arithmetic is written again with Python floats and explicit loops, so that an indexing or
transposition slip in the vectorised model shows up as a disagreement.
"""
import math


def _dot(a, b):
    return math.fsum(x * y for x, y in zip(a, b))


def _matvec(W, x):                      # W [out][in]
    return [_dot(row, x) for row in W]


def _rmsnorm(x, g, eps):
    ms = math.fsum(v * v for v in x) / len(x)
    r = 1.0 / math.sqrt(ms + eps)
    return [v * r * gi for v, gi in zip(x, g)]


def _rope(vec, p, theta):
    dh = len(vec)
    half = dh // 2
    out = [0.0] * dh
    for i in range(half):
        ang = p * theta ** (-2.0 * i / dh)
        c, s = math.cos(ang), math.sin(ang)
        out[i] = vec[i] * c - vec[i + half] * s
        out[i + half] = vec[i + half] * c + vec[i] * s
    return out


def step_logits(model, weights, tokens, active_history, hist_k, hist_v, t):
    """Logits of the rows active at step t for ONE sequence.

    tokens: ids of the sequence as input to step t. active_history[s] = active positions of step
    s (s <= t). hist_k[s][l][p] / hist_v[s][l][p] = rows computed at step s; this call appends the
    entries of step t. Returns {position: [V logits]}."""
    L = len(tokens)
    Hq, Hkv, dh, d = model.n_q_heads, model.n_kv_heads, model.head_dim, model.d_model
    group = Hq // Hkv
    act = active_history[t]
    E = weights.embed().tolist()
    h = {p: list(E[tokens[p]]) for p in act}
    hist_k.append([dict() for _ in range(model.n_layers)])
    hist_v.append([dict() for _ in range(model.n_layers)])

    def last_computed(p):
        for s in range(t, -1, -1):
            if p in active_history[s]:
                return s
        raise KeyError("position never computed")

    for l in range(model.n_layers):
        w = {k: v.tolist() for k, v in weights.layer(l).items()}
        q = {}
        for p in act:
            a = _rmsnorm(h[p], w["norm1"], model.rms_eps)
            qf, kf, vf = _matvec(w["wq"], a), _matvec(w["wk"], a), _matvec(w["wv"], a)
            q[p] = [_rope(qf[i * dh:(i + 1) * dh], p, model.rope_theta) for i in range(Hq)]
            hist_k[t][l][p] = [_rope(kf[i * dh:(i + 1) * dh], p, model.rope_theta) for i in range(Hkv)]
            hist_v[t][l][p] = [vf[i * dh:(i + 1) * dh] for i in range(Hkv)]
        # K_t^I, V_t^I: cached rows of I \ A_t joined with the fresh rows of A_t (Eq. 4)
        K_I = [hist_k[last_computed(p)][l][p] for p in range(L)]
        V_I = [hist_v[last_computed(p)][l][p] for p in range(L)]
        for p in act:
            o = []
            for hq in range(Hq):
                kv = hq // group
                sc = [_dot(q[p][hq], K_I[j][kv]) / math.sqrt(dh) for j in range(L)]
                mx = max(sc)
                e = [math.exp(s - mx) for s in sc]
                z = math.fsum(e)
                o += [math.fsum(e[j] / z * V_I[j][kv][c] for j in range(L)) for c in range(dh)]
            att = _matvec(w["wo"], o)
            h[p] = [x + y for x, y in zip(h[p], att)]
            m = _rmsnorm(h[p], w["norm2"], model.rms_eps)
            g, u = _matvec(w["w_gate"], m), _matvec(w["w_up"], m)
            f = [gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)]
            dn = _matvec(w["w_down"], f)
            h[p] = [x + y for x, y in zip(h[p], dn)]
    head = weights.lm_head().tolist()
    gf = weights.final_norm().tolist()
    return {p: _matvec(head, _rmsnorm(h[p], gf, model.rms_eps)) for p in act}
