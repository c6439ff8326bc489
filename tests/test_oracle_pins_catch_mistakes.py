"""Do the pins bite? Each case plants one plausible mistake in the oracle (a dropped term, a wrong
sign or index, a swapped operand, an off-by-one in the schedule), on the CPU, and requires that at
least one pin of test_oracle_model / test_oracle_schedule then fails. The oracle itself is left as
it was when a case ends."""
import math
import numpy as np
import pytest
from dkv_inputs.configs import DECODE, GREEDY, PD
from oracle import model as M, sampler as SA, schedule as S
import test_oracle_model as TM
import test_oracle_schedule as TS


def _caught_by(pins):
    """Names of the pins that fail with the mistake in place."""
    failed = []
    for pin in pins:
        fn, args = (pin, ()) if callable(pin) else (pin[0], pin[1:])
        try:
            fn(*args)
        except AssertionError:
            failed.append(fn.__name__)
        except Exception as e:                      # a NaN / index error caused by the mistake counts too
            failed.append(f"{fn.__name__} ({type(e).__name__})")
    return failed


# ---- mistakes in the arithmetic (oracle.model)

def _attention_without_scale(q, K, V, group):
    n, Hq, dh = q.shape
    out = np.empty_like(q)
    for h in range(Hq):
        out[:, h, :] = M.softmax(q[:, h, :] @ K[h // group].T, axis=-1) @ V[h // group]
    return out


def _attention_values_from_keys(q, K, V, group):
    n, Hq, dh = q.shape
    out = np.empty_like(q)
    for h in range(Hq):
        out[:, h, :] = M.softmax(q[:, h, :] @ K[h // group].T / np.sqrt(dh), axis=-1) @ K[h // group]
    return out


def _attention_interleaved_groups(q, K, V, group):
    n, Hq, dh = q.shape
    Hkv = K.shape[0]
    out = np.empty_like(q)
    for h in range(Hq):
        out[:, h, :] = M.softmax(q[:, h, :] @ K[h % Hkv].T / np.sqrt(dh), axis=-1) @ V[h % Hkv]
    return out


def _attention_causal(q, K, V, group):
    """A mask where the method has none: query row i sees only the first i + 1 stored positions."""
    n, Hq, dh = q.shape
    out = np.empty_like(q)
    for h in range(Hq):
        s = q[:, h, :] @ K[h // group].T / np.sqrt(dh)
        s = np.where(np.arange(s.shape[1])[None, :] <= np.arange(n)[:, None], s, -np.inf)
        out[:, h, :] = M.softmax(s, axis=-1) @ V[h // group]
    return out


def _rmsnorm_without_root(h, gain, eps):
    h = np.asarray(h, dtype=np.float64)
    return h / (np.mean(h * h, axis=-1, keepdims=True) + eps) * np.asarray(gain, dtype=np.float64)


def _rmsnorm_centred(h, gain, eps):
    h = np.asarray(h, dtype=np.float64)
    c = h - np.mean(h, axis=-1, keepdims=True)
    return c / np.sqrt(np.mean(c * c, axis=-1, keepdims=True) + eps) * np.asarray(gain, dtype=np.float64)


def _silu_wrong_sign(x):
    return x / (1.0 + np.exp(x))


def _rope_with(freq_exponent_scale=2.0, pos_shift=0, adjacent_pairs=False, second_sign=1.0):
    def rope(x, pos, theta):
        x = np.asarray(x, dtype=np.float64)
        dh = x.shape[-1]
        half = dh // 2
        inv_freq = theta ** (-freq_exponent_scale * np.arange(half, dtype=np.float64) / dh)
        ang = (np.asarray(pos, dtype=np.float64)[:, None] + pos_shift) * inv_freq[None, :]
        c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
        if adjacent_pairs:
            x1, x2 = x[..., 0::2], x[..., 1::2]
            out = np.empty_like(x)
            out[..., 0::2], out[..., 1::2] = x1 * c - x2 * s, x2 * c + x1 * s
            return out
        x1, x2 = x[..., :half], x[..., half:]
        return np.concatenate([x1 * c - x2 * s, x2 * c + second_sign * x1 * s], axis=-1)
    return rope


def _softmax_without_normalisation(s, axis=-1):
    return np.exp(s - np.max(s, axis=axis, keepdims=True))


ARITHMETIC = [
    ("attention: 1/sqrt(d_h) dropped", "attention", _attention_without_scale,
     [TM.test_attention_matches_explicit_loops_and_gqa_is_head_sharing]),
    ("attention: values taken from K", "attention", _attention_values_from_keys,
     [TM.test_attention_special_cases, TM.test_attention_matches_explicit_loops_and_gqa_is_head_sharing]),
    ("attention: query head h reads kv head h mod H_kv", "attention", _attention_interleaved_groups,
     [TM.test_attention_matches_explicit_loops_and_gqa_is_head_sharing]),
    ("attention: a causal mask", "attention", _attention_causal,
     [TM.test_attention_special_cases, TM.test_attention_matches_explicit_loops_and_gqa_is_head_sharing]),
    ("RMSNorm: square root dropped", "rmsnorm", _rmsnorm_without_root, [TM.test_rmsnorm_closed_forms]),
    ("RMSNorm: mean subtracted (LayerNorm)", "rmsnorm", _rmsnorm_centred, [TM.test_rmsnorm_closed_forms]),
    ("SiLU: sigmoid of -x", "silu", _silu_wrong_sign, [TM.test_silu_values]),
    ("RoPE: exponent i/d_h instead of 2i/d_h", "rope", _rope_with(freq_exponent_scale=1.0),
     [TM.test_rope_is_a_rotation_by_position_times_frequency]),
    ("RoPE: positions counted from 1", "rope", _rope_with(pos_shift=1),
     [TM.test_rope_is_a_rotation_by_position_times_frequency]),
    ("RoPE: neighbouring elements paired", "rope", _rope_with(adjacent_pairs=True),
     [TM.test_rope_is_a_rotation_by_position_times_frequency]),
    ("RoPE: sign of one sine term", "rope", _rope_with(second_sign=-1.0),
     [TM.test_rope_is_a_rotation_by_position_times_frequency,
      TM.test_rope_keeps_norms_and_makes_scores_depend_on_relative_position]),
    ("softmax: not normalised", "softmax", _softmax_without_normalisation,
     [TM.test_softmax_rows_sum_to_one_and_are_shift_invariant]),
]


@pytest.mark.parametrize("what,name,wrong,pins", ARITHMETIC, ids=[a[0] for a in ARITHMETIC])
def test_arithmetic_mistake_fails_a_pin(monkeypatch, what, name, wrong, pins):
    monkeypatch.setattr(M, name, wrong)
    assert _caught_by(pins), f"no pin notices: {what}"


# ---- mistakes in the forward pass over the store

def test_storing_keys_before_the_rotation_fails_a_pin(monkeypatch):
    """Cached K must be the rotated one: with the rotation applied to Q only, scores depend on absolute
    positions and the two cache formulations / the literal Eq. 4 assembly no longer see what a cache-free
    pass sees."""
    real = M.rope
    calls = {"n": 0}

    def rope_q_only(x, pos, theta):
        calls["n"] += 1
        return real(x, pos, theta) if calls["n"] % 2 == 1 else np.asarray(x, dtype=np.float64)   # q first, then k
    monkeypatch.setattr(M, "rope", rope_q_only)
    assert _caught_by([TM.test_rope_keeps_norms_and_makes_scores_depend_on_relative_position,
                       (TM.test_one_layer_model_with_one_step_delay_reproduces_full_recomputation, 4),
                       TM.test_attn_update_scatters_then_attends_over_everything])


# ---- mistakes in the schedule (oracle.schedule)

def _decode_without_previous_commit(run, t, masked, d_prev, d_cur=None, forced_scope=None):
    """Eq. 3 where Eq. 4 is asked for: the one-step delay dropped."""
    if run.variant in (DECODE, PD) and t > 0 and forced_scope is None and not S.is_refresh_step(run, t):
        return sorted(p for p in range(run.seq_len) if masked[p])
    return _REAL_SELECT(run, t, masked, d_prev, d_cur, forced_scope)


def _refresh_one_step_late(run, t):
    return t % run.refresh_interval == 1 % run.refresh_interval


def _window_floor_ceil_swapped(center, w, L):
    return [p for p in range(center - math.floor(w / 2), center + math.ceil(w / 2) + 1) if 0 <= p < L]


def _window_unclipped(center, w, L):
    return list(range(center - math.ceil(w / 2), center + math.floor(w / 2) + 1))


def _block_of_previous_step(run, t):
    j = max(t - 1, 0) // run.steps_per_block
    lo = run.prompt_len + j * run.block_len
    return lo, lo + run.block_len


def _pd_refreshes_everything(run, t, masked, d_prev, d_cur=None, forced_scope=None):
    if run.variant == PD and t > 0 and forced_scope is None and S.is_refresh_step(run, t):
        return list(range(run.seq_len))
    return _REAL_SELECT(run, t, masked, d_prev, d_cur, forced_scope)


def _greedy_forgets_the_previous_commit(run, t, masked, d_prev, d_cur=None, forced_scope=None):
    if run.variant == GREEDY:
        return _REAL_SELECT(run, t, masked, [], d_cur, forced_scope)
    return _REAL_SELECT(run, t, masked, d_prev, d_cur, forced_scope)


_REAL_SELECT = S._select_unshifted

SCHEDULE = [
    ("Decode: D_{t-1} not recomputed", "_select_unshifted", _decode_without_previous_commit,
     [TS.test_decode_active_set_is_masked_plus_previous_commit,
      (TM.test_one_layer_model_with_one_step_delay_reproduces_full_recomputation, 4)]),
    ("refresh one step late", "is_refresh_step", _refresh_one_step_late,
     [TS.test_refresh_steps_and_blocks, (TS.test_cache_ratio_of_the_benchmark_schedules, 2, 0.655)]),
    ("window: floor and ceiling swapped", "window", _window_floor_ceil_swapped,
     [TS.test_window_formula_and_clipping]),
    ("window: not clipped to the sequence", "window", _window_unclipped, [TS.test_window_formula_and_clipping]),
    ("candidates from the previous step's block", "block_range", _block_of_previous_step,
     [TS.test_refresh_steps_and_blocks]),
    ("PD refresh recomputes the prompt too", "_select_unshifted", _pd_refreshes_everything,
     [TS.test_prefill_and_pd_active_sets, (TS.test_cache_ratio_of_the_benchmark_schedules, 4, 0.788)]),
    ("Greedy: D_{t-1} left out although include_prev is set", "_select_unshifted",
     _greedy_forgets_the_previous_commit,
     [TS.test_greedy_active_set_membership,
      (TM.test_one_layer_greedy_is_exact_only_when_the_previous_commit_is_recomputed, 1)]),
]


@pytest.mark.parametrize("what,name,wrong,pins", SCHEDULE, ids=[a[0] for a in SCHEDULE])
def test_schedule_mistake_fails_a_pin(monkeypatch, what, name, wrong, pins):
    monkeypatch.setattr(S, name, wrong)
    assert _caught_by(pins), f"no pin notices: {what}"


# ---- mistakes in the sampler

def _predict_without_exclusion(logits, mask_id):
    lg = np.asarray(logits, dtype=np.float64).astype(np.float32)
    tok = np.argmax(lg, axis=1)
    top = lg[np.arange(lg.shape[0]), tok].astype(np.float64)
    conf = 1.0 / np.sum(np.exp(lg.astype(np.float64) - top[:, None]), axis=1)
    return tok.astype(np.int32), conf.astype(np.float32)


def _predict_highest_id_on_ties(logits, mask_id):
    lg = np.asarray(logits, dtype=np.float64).astype(np.float32)
    lg[:, mask_id] = -np.inf
    tok = lg.shape[1] - 1 - np.argmax(lg[:, ::-1], axis=1)
    top = lg[np.arange(lg.shape[0]), tok].astype(np.float64)
    conf = 1.0 / np.sum(np.exp(lg.astype(np.float64) - top[:, None]), axis=1)
    return tok.astype(np.int32), conf.astype(np.float32)


def _top_k_least_confident(positions, conf, k):
    order = sorted(range(len(positions)), key=lambda i: (float(conf[i]), positions[i]))
    return [positions[i] for i in order[:k]]


def _top_k_higher_position_on_ties(positions, conf, k):
    order = sorted(range(len(positions)), key=lambda i: (-float(conf[i]), -positions[i]))
    return [positions[i] for i in order[:k]]


SAMPLER = [
    ("a position may decode to the MASK token", "predict", _predict_without_exclusion,
     [TM.test_predict_excludes_mask_breaks_ties_low_and_reports_softmax_max]),
    ("arg max: highest id on ties", "predict", _predict_highest_id_on_ties,
     [TM.test_predict_excludes_mask_breaks_ties_low_and_reports_softmax_max]),
    ("top-k keeps the least confident", "top_k_positions", _top_k_least_confident,
     [TM.test_top_k_prefers_confidence_then_lower_position]),
    ("top-k: higher position on ties", "top_k_positions", _top_k_higher_position_on_ties,
     [TM.test_top_k_prefers_confidence_then_lower_position]),
]


@pytest.mark.parametrize("what,name,wrong,pins", SAMPLER, ids=[a[0] for a in SAMPLER])
def test_sampler_mistake_fails_a_pin(monkeypatch, what, name, wrong, pins):
    monkeypatch.setattr(SA, name, wrong)
    assert _caught_by(pins), f"no pin notices: {what}"


def test_the_unmutated_oracle_passes_every_pin_used_here():
    pins = {id(p if callable(p) else p[0]): p for group in (ARITHMETIC, SCHEDULE, SAMPLER) for case in group
            for p in case[3]}
    assert _caught_by(list(pins.values())) == []
