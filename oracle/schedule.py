"""Which positions are recomputed at each denoising step (oracle; test infrastructure).

Notation of Sec. 3.3-3.4: I = all positions, M = masked (not yet finalised)
positions, D_t = positions committed at step t, A_t = rows fed through the
transformer at step t. Positions are 0-based; the generated region is
[prompt_len, seq_len).
"""
import math
from dkv_inputs.configs import (DECODE, GREEDY, PREFILL, PD, CENTER_CUR, CENTER_PREV,
                                SCOPE_ALL, SCOPE_GEN)


def validate_run(run):
    """Schedules this build accepts: whole blocks, the same number of steps per
    block, the same number of commits per step."""
    ok = (run.batch >= 1 and run.prompt_len >= 0 and run.gen_len >= 1 and run.steps >= 1
          and run.block_len >= 1 and run.refresh_interval >= 1
          and run.gen_len % run.block_len == 0
          and run.steps % (run.gen_len // run.block_len) == 0
          and run.block_len % (run.steps // (run.gen_len // run.block_len)) == 0
          and (not run.shift_logits or run.prompt_len >= 1))
    return ok


def is_refresh_step(run, t):
    """Cache refresh (Sec. 3.3, "Cache Refreshing Mechanism"): every N-th step on a
    global 0-based counter; step 0 has no cache yet so it always recomputes."""
    return t % run.refresh_interval == 0


def block_range(run, t):
    """Semi-autoregressive block [lo, hi) whose positions may be committed at step t."""
    j = t // run.steps_per_block
    lo = run.prompt_len + j * run.block_len
    return lo, lo + run.block_len


def window(center, w, L):
    """Local window of Sec. 3.4: [c - ceil(w/2), c + floor(w/2)], clipped to the sequence."""
    lo = center - math.ceil(w / 2)
    hi = center + math.floor(w / 2)
    return [p for p in range(lo, hi + 1) if 0 <= p < L]


def refresh_scope_positions(run, scope):
    L = run.seq_len
    if scope == SCOPE_ALL:
        return list(range(L))
    if scope == SCOPE_GEN:
        return list(range(run.prompt_len, L))
    raise ValueError("unknown refresh scope")


def _select_unshifted(run, t, masked, d_prev, d_cur=None, forced_scope=None):
    """Active positions of ONE sequence at step t without the extra rows of shifted logits.

    masked : sequence of L booleans, the mask set in the INPUT of step t (M_t).
    d_prev : positions committed at step t-1 (D_{t-1}; empty at t = 0).
    d_cur  : positions that step t will commit (D_t); known beforehand only under a
             predefined decode order, required by the Greedy variant.
    forced_scope : an explicit, out-of-schedule refresh request for this step.

    Decode (Eq. 4): queries are M_{t-1} = M_t + D_{t-1}: everything still masked plus what
    was decoded one step ago, whose K/V are recomputed from the decoded token before being
    reused (one-step delay). With run.delay == 0 (Eq. 3) only M_t is recomputed.
    Refresh: the cached set is emptied, so all of I is recomputed.
    Prefill: the prompt is computed once at step 0; the generated region is always recomputed.
    PD: Prefill for the prompt, Decode (with refresh of the generated region only) for the rest.
    Greedy (Sec. 3.4): D_t, D_{t-1} and a local window, between full refreshes.
    """
    L = run.seq_len
    P = run.prompt_len
    assert len(masked) == L
    if forced_scope is not None:
        return refresh_scope_positions(run, forced_scope)
    if t == 0:
        return list(range(L))
    refresh = is_refresh_step(run, t)
    v = run.variant
    if v == PREFILL:
        return list(range(P, L))
    if refresh:
        return list(range(P, L)) if v == PD else list(range(L))
    if v in (DECODE, PD):
        act = {p for p in range(L) if masked[p]}
        if run.delay:
            act |= set(d_prev)
        return sorted(act)
    if v == GREEDY:
        assert d_cur is not None, "Greedy needs the decode order ahead of the forward pass"
        act = set(d_cur)
        if run.include_prev:
            act |= set(d_prev)
        centers = d_cur if run.window_center == CENTER_CUR else d_prev
        if run.window > 0:
            for c in centers:
                act |= set(window(c, run.window, L))
        return sorted(p for p in act if 0 <= p < L)
    raise ValueError("unknown variant")


def select_active(run, t, masked, d_prev, d_cur=None, forced_scope=None):
    """Active positions of ONE sequence at step t, sorted ascending, unique (see _select_unshifted
    for the sets of each variant).

    With run.shift_logits (a model adapted from an autoregressive one, Appendix B: the output at
    position i is the distribution of token i + 1, and K/V are cached unshifted, at the token's own
    position) the row that predicts a candidate q is q - 1, so q - 1 joins the active set for every
    position q that may be committed at this step."""
    act = _select_unshifted(run, t, masked, d_prev, d_cur, forced_scope)
    if run.shift_logits:
        extra = {q - 1 for q in candidates(run, t, act, masked)}
        assert all(p >= 0 for p in extra)
        act = sorted(set(act) | extra)
    return act


def step_candidates(run, t, masked, d_prev, d_cur=None, forced_scope=None):
    """Positions whose prediction may be committed at step t: members of the variant's own set (the
    rows added for shifted logits do not count) that are still masked and lie in the block."""
    return candidates(run, t, _select_unshifted(run, t, masked, d_prev, d_cur, forced_scope), masked)


def candidates(run, t, active, masked):
    """Rows whose prediction may be committed at step t: active, still masked, in the block."""
    lo, hi = block_range(run, t)
    return [p for p in active if masked[p] and lo <= p < hi]


def cache_ratio(active_sizes, L):
    """Mean fraction of positions whose K/V are reused rather than recomputed
    (the cache-ratio metric of Sec. 4.1, reading the reused count as L - |A_t|)."""
    return sum((L - a) / L for a in active_sizes) / len(active_sizes)


def reorder_map(unmasked_prev, unmasked_next, L):
    """Index bookkeeping of concat_reorder (Appendix A).

    The layout puts cached (unmasked) positions on the left and recomputed ones on the
    right. Returns (layout_prev, layout_next, mapping, take): mapping[i] is where the
    position layout_next[i] sits inside layout_prev, and take = the first
    len(unmasked_next) entries, i.e. the rows to keep as next step's cache."""
    up, un = sorted(unmasked_prev), sorted(unmasked_next)
    layout_prev = up + [p for p in range(L) if p not in set(up)]
    layout_next = un + [p for p in range(L) if p not in set(un)]
    where = {p: i for i, p in enumerate(layout_prev)}
    mapping = [where[p] for p in layout_next]
    return layout_prev, layout_next, mapping, mapping[:len(un)]
