"""The T-step denoising loop with the delayed K/V cache (oracle; test infrastructure).

Per step: pick the active set, run the partial forward, turn the candidate rows' logits into
(confidence, token), commit k positions, and hand the new mask set to the next step
(sampling process of Sec. 3.1; Eq. 4; Algorithm 1).
"""
from dataclasses import dataclass, field
import numpy as np
from dkv_inputs.configs import CONFIDENCE, RANDOM_ORDER, GREEDY
from . import schedule as S
from .model import KVStore, forward_active, logits_of


def predict(logits, mask_id):
    """(token, confidence) per row. The MASK id can never be predicted. Decisions are taken on
    float32 logits (the precision the device path holds them in): token = arg max, lowest id on
    ties; confidence = its softmax probability, returned as float32."""
    l = np.asarray(logits, dtype=np.float64).astype(np.float32)
    if np.isnan(l).any():
        raise FloatingPointError("NaN logits")
    l[:, mask_id] = -np.inf
    tok = np.argmax(l, axis=1)
    top = l[np.arange(l.shape[0]), tok].astype(np.float64)
    conf = 1.0 / np.sum(np.exp(l.astype(np.float64) - top[:, None]), axis=1)
    return tok.astype(np.int32), conf.astype(np.float32)


def top_k_positions(positions, conf, k):
    """The k candidate positions of highest confidence, best first; ties go to the lower position."""
    order = sorted(range(len(positions)), key=lambda i: (-float(conf[i]), positions[i]))
    return [positions[i] for i in order[:k]]


@dataclass
class StepLog:
    t: int
    active: list                      # per sequence: sorted positions
    cand: list                        # per sequence: candidate positions
    cand_tok: list                    # per sequence: int32 [n_cand]
    cand_conf: list                   # per sequence: float32 [n_cand]
    cand_logits: list                 # per sequence: float64 [n_cand, V] or None
    pos: np.ndarray                   # [B, k] committed positions
    tok: np.ndarray                   # [B, k] committed tokens
    conf: np.ndarray                  # [B, k] their confidences
    hidden: np.ndarray = None         # [R, d] final hidden rows (before final norm), optional


@dataclass
class RunState:
    tokens: np.ndarray                # [B, L]
    masked: np.ndarray                # [B, L] bool
    store: KVStore
    d_prev: list                      # per sequence: positions committed at the previous step
    logs: list = field(default_factory=list)


def init_state(model, run, prompt):
    B, L, P = run.batch, run.seq_len, run.prompt_len
    tokens = np.full((B, L), model.mask_id, dtype=np.int32)
    tokens[:, :P] = prompt
    masked = np.zeros((B, L), dtype=bool)
    masked[:, P:] = True
    return RunState(tokens, masked, KVStore(model, B, L), [[] for _ in range(B)])


def denoise_step(model, weights, run, st, t, order=None, forced=None, forced_scope=None,
                 keep_logits=False, keep_hidden=False, head_all_rows=False):
    """Advance the state by one denoising step and return its StepLog.

    order  : [B, G] predefined decode order (RANDOM_ORDER runs).
    forced : (pos [B,k], tok [B,k]) committed instead of the step's own choice (teacher forcing).
    """
    B, k = run.batch, run.k_per_step
    d_cur = [None] * B
    if run.remask == RANDOM_ORDER:
        d_cur = [[int(p) for p in order[b, t * k:(t + 1) * k]] for b in range(B)]
    active = [S.select_active(run, t, st.masked[b], st.d_prev[b], d_cur[b], forced_scope)
              for b in range(B)]
    h = forward_active(model, weights, st.tokens, active, st.store, t)

    off = np.concatenate([[0], np.cumsum([len(a) for a in active])]).astype(int)
    cand, cand_tok, cand_conf, cand_logits = [], [], [], []
    pos = np.zeros((B, k), dtype=np.int32)
    tok = np.zeros((B, k), dtype=np.int32)
    conf = np.zeros((B, k), dtype=np.float32)
    for b in range(B):
        c = S.step_candidates(run, t, st.masked[b], st.d_prev[b], d_cur[b], forced_scope)
        # the row whose output is the distribution of position p: p itself, or p - 1 under shifted logits
        src = [active[b].index(p - (1 if run.shift_logits else 0)) for p in c]
        rows = [off[b] + i for i in src]
        if head_all_rows:
            all_logits = logits_of(model, weights, h[off[b]:off[b + 1]])
            lg = all_logits[src]
        else:
            lg = logits_of(model, weights, h[rows])
        tk, cf = predict(lg, model.mask_id)
        cand.append(c); cand_tok.append(tk); cand_conf.append(cf)
        cand_logits.append(lg if keep_logits else None)
        if run.remask == CONFIDENCE:
            chosen = top_k_positions(c, cf, k)
        else:
            chosen = d_cur[b]
            assert all(p in c for p in chosen), "ordered position is not a candidate of its step"
        assert len(chosen) == k
        for j, p in enumerate(chosen):
            i = c.index(p)
            pos[b, j], tok[b, j], conf[b, j] = p, tk[i], cf[i]
    if forced is not None:
        fpos, ftok = forced
        for b in range(B):
            for j in range(k):
                p = int(fpos[b, j])
                assert p in cand[b], "forced position is not a candidate of its step"
                pos[b, j], tok[b, j] = p, int(ftok[b, j])
                conf[b, j] = cand_conf[b][cand[b].index(p)]
    for b in range(B):
        for j in range(k):
            st.tokens[b, pos[b, j]] = tok[b, j]
            st.masked[b, pos[b, j]] = False
        st.d_prev[b] = [int(p) for p in pos[b]]
    log = StepLog(t, active, cand, cand_tok, cand_conf, cand_logits, pos, tok, conf,
                  h if keep_hidden else None)
    st.logs.append(log)
    return log


def generate(model, weights, run, prompt, order=None, forced=None, forced_scopes=None,
             keep_logits=False, keep_hidden=False, steps=None):
    """Run `steps` (default: all T) denoising steps from the fully masked state."""
    assert S.validate_run(run)
    st = init_state(model, run, prompt)
    for t in range(run.steps if steps is None else steps):
        denoise_step(model, weights, run, st, t, order=order,
                     forced=None if forced is None else forced[t],
                     forced_scope=None if forced_scopes is None else forced_scopes.get(t),
                     keep_logits=keep_logits, keep_hidden=keep_hidden)
    return st
