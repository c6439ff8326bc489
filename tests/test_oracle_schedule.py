"""Pins of the oracle's schedule: printed worked example, closed forms, invariants."""
import math
import os
import numpy as np
import pytest
import dkv_inputs as D
from dkv_inputs.configs import (RunShape, DECODE, GREEDY, PREFILL, PD, RANDOM_ORDER, CENTER_CUR,
                                CENTER_PREV, SCOPE_ALL, SCOPE_GEN)
from oracle import schedule as S
from helpers import simulate_schedule

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        out[k] = [int(x) for x in v]
    return out


def test_appendix_a_worked_example():
    g = _read_golden("appendix_a_reorder.txt")
    lp, ln, mapping, take = S.reorder_map(g["unmasked_prev"], g["unmasked_next"], g["seq_len"][0])
    assert lp == g["layout_prev"]
    assert ln == g["layout_next"]
    assert mapping == g["mapping"]
    assert take == g["take"]


def test_reorder_map_is_a_permutation_and_picks_the_right_rows():
    rng = np.random.default_rng(3)
    for _ in range(50):
        L = int(rng.integers(2, 20))
        perm = rng.permutation(L)
        n0 = int(rng.integers(0, L))
        n1 = int(rng.integers(n0, L + 1))
        up, un = sorted(perm[:n0].tolist()), sorted(perm[:n1].tolist())
        lp, ln, mapping, take = S.reorder_map(up, un, L)
        assert sorted(mapping) == list(range(L))
        assert [lp[i] for i in mapping] == ln
        assert [lp[i] for i in take] == un


def test_window_formula_and_clipping():
    # [c - ceil(w/2), c + floor(w/2)]
    assert S.window(10, 4, 100) == [8, 9, 10, 11, 12]
    assert S.window(10, 3, 100) == [8, 9, 10, 11]
    assert S.window(10, 0, 100) == [10]
    assert S.window(0, 4, 100) == [0, 1, 2]
    assert S.window(99, 4, 100) == [97, 98, 99]
    assert S.window(10, 6, 100) == list(range(7, 14))


def test_refresh_steps_and_blocks():
    run = RunShape(batch=1, prompt_len=4, gen_len=8, steps=8, block_len=4, refresh_interval=3)
    assert [t for t in range(8) if S.is_refresh_step(run, t)] == [0, 3, 6]
    assert [S.block_range(run, t) for t in (0, 3, 4, 7)] == [(4, 8), (4, 8), (8, 12), (8, 12)]
    assert run.k_per_step == 1 and run.steps_per_block == 4
    run2 = RunShape(batch=1, prompt_len=4, gen_len=8, steps=4, block_len=4, refresh_interval=3)
    assert run2.k_per_step == 2 and run2.steps_per_block == 2


def test_validate_run_rejects_ragged_schedules():
    ok = RunShape(batch=1, prompt_len=4, gen_len=8, steps=8, block_len=4, refresh_interval=3)
    assert S.validate_run(ok)
    assert not S.validate_run(RunShape(1, 4, 8, 8, 3, 3))     # blocks do not tile the region
    assert not S.validate_run(RunShape(1, 4, 8, 3, 4, 3))     # steps not a multiple of blocks
    assert S.validate_run(RunShape(1, 4, 12, 6, 4, 3))        # 3 blocks x 2 steps, 2 commits a step
    assert not S.validate_run(RunShape(1, 4, 8, 6, 4, 3))     # 3 steps per block do not split 4 positions
    assert not S.validate_run(RunShape(1, 4, 8, 8, 4, 0))     # refresh interval must be >= 1


def test_decode_active_set_is_masked_plus_previous_commit():
    run = RunShape(batch=1, prompt_len=3, gen_len=5, steps=5, block_len=5, refresh_interval=100)
    masked = [False, False, False, True, False, True, True, False]
    assert S.select_active(run, 2, masked, [4]) == [3, 4, 5, 6]
    run0 = RunShape(batch=1, prompt_len=3, gen_len=5, steps=5, block_len=5, refresh_interval=100, delay=0)
    assert S.select_active(run0, 2, masked, [4]) == [3, 5, 6]
    assert S.select_active(run, 0, [False] * 3 + [True] * 5, []) == list(range(8))
    assert S.select_active(run, 2, masked, [4], forced_scope=SCOPE_GEN) == [3, 4, 5, 6, 7]
    assert S.select_active(run, 2, masked, [4], forced_scope=SCOPE_ALL) == list(range(8))


def test_shifted_logits_add_the_row_before_every_candidate():
    # Appendix B: a model adapted from an autoregressive one predicts token q at row q - 1, so that row is
    # recomputed whenever q may be committed; nothing else changes.
    masked = [False, False, False, True, False, True, True, False]
    run = RunShape(batch=1, prompt_len=3, gen_len=5, steps=5, block_len=5, refresh_interval=100, shift_logits=1)
    # masked 3, 5, 6 (+ previous commit 4): candidates 3, 5, 6 need rows 2, 4, 5 -> 2 joins
    assert S.select_active(run, 2, masked, [4]) == [2, 3, 4, 5, 6]
    nodelay = RunShape(batch=1, prompt_len=3, gen_len=5, steps=5, block_len=5, refresh_interval=100, delay=0,
                       shift_logits=1)
    assert S.select_active(nodelay, 2, masked, [4]) == [2, 3, 4, 5, 6]          # 4 returns as the row before 5
    # two blocks of 4: only candidates of the current block pull their predecessor in
    m2 = [False, False, True, False, True, True, True, True, True, True]
    blocks = RunShape(batch=1, prompt_len=2, gen_len=8, steps=8, block_len=4, refresh_interval=100, shift_logits=1)
    assert S.select_active(blocks, 1, m2, []) == [1, 2, 3, 4, 5, 6, 7, 8, 9]     # candidates 2, 4, 5: rows 1, 3
    plain = RunShape(batch=1, prompt_len=2, gen_len=8, steps=8, block_len=4, refresh_interval=100)
    assert S.select_active(plain, 1, m2, []) == [2, 4, 5, 6, 7, 8, 9]
    # generated-region-only sets (Prefill, PD refresh) reach one row into the prompt
    pre = RunShape(batch=1, prompt_len=3, gen_len=5, steps=5, block_len=5, refresh_interval=2, variant=PREFILL,
                   shift_logits=1)
    assert S.select_active(pre, 1, masked, [4]) == [2, 3, 4, 5, 6, 7]
    assert not S.validate_run(RunShape(batch=1, prompt_len=0, gen_len=4, steps=4, block_len=4, refresh_interval=2,
                                       shift_logits=1))
    # Greedy: the added row may itself be masked and in the block, but it is not a candidate of the step
    gr = RunShape(batch=1, prompt_len=2, gen_len=8, steps=8, block_len=8, refresh_interval=100, variant=GREEDY,
                  window=0, remask=RANDOM_ORDER, shift_logits=1)
    m3 = [False, False, True, True, True, True, True, True, True, True]
    assert S.select_active(gr, 1, m3, [], d_cur=[6]) == [5, 6]
    assert S.step_candidates(gr, 1, m3, [], d_cur=[6]) == [6]


def test_prefill_and_pd_active_sets():
    masked = [False, False, False, True, False, True, True, False]
    pre = RunShape(batch=1, prompt_len=3, gen_len=5, steps=5, block_len=5, refresh_interval=2, variant=PREFILL)
    pd = RunShape(batch=1, prompt_len=3, gen_len=5, steps=5, block_len=5, refresh_interval=2, variant=PD)
    assert S.select_active(pre, 0, [False] * 3 + [True] * 5, []) == list(range(8))
    assert S.select_active(pre, 1, masked, [4]) == [3, 4, 5, 6, 7]
    assert S.select_active(pre, 2, masked, [4]) == [3, 4, 5, 6, 7]
    assert S.select_active(pd, 0, [False] * 3 + [True] * 5, []) == list(range(8))
    assert S.select_active(pd, 1, masked, [4]) == [3, 4, 5, 6]
    assert S.select_active(pd, 2, masked, [4]) == [3, 4, 5, 6, 7]      # refresh: generated region only


def test_greedy_active_set_membership():
    base = dict(batch=1, prompt_len=10, gen_len=20, steps=20, block_len=20, refresh_interval=100,
                variant=GREEDY, remask=RANDOM_ORDER)
    masked = [False] * 10 + [True] * 20
    run = RunShape(window=4, window_center=CENTER_CUR, include_prev=1, **base)
    assert S.select_active(run, 3, masked, [25], [12]) == [10, 11, 12, 13, 14, 25]
    run = RunShape(window=4, window_center=CENTER_PREV, include_prev=1, **base)
    assert S.select_active(run, 3, masked, [25], [12]) == [12, 23, 24, 25, 26, 27]
    run = RunShape(window=4, window_center=CENTER_CUR, include_prev=0, **base)
    assert S.select_active(run, 3, masked, [25], [12]) == [10, 11, 12, 13, 14]
    run = RunShape(window=0, include_prev=1, **base)
    assert S.select_active(run, 3, masked, [25], [12]) == [12, 25]
    run = RunShape(window=4, include_prev=1, **base)
    assert S.select_active(run, 3, masked, [28], [29]) == [27, 28, 29]   # clipped at the end
    assert S.select_active(run, 3, masked, [0 + 10], [11]) == [9, 10, 11, 12, 13]  # window reaches the prompt
    assert S.select_active(run, 0, masked, [], [12]) == list(range(30))


def _closed_form_sizes(run):
    """|A_t| the schedule implies (Decode / PD / Prefill), from |M_t| = G - t*k."""
    L, P, G, k = run.seq_len, run.prompt_len, run.gen_len, run.k_per_step
    out = []
    for t in range(run.steps):
        if t == 0:
            out.append(L)
        elif run.variant == PREFILL:
            out.append(G)
        elif t % run.refresh_interval == 0:
            out.append(G if run.variant == PD else L)
        else:
            out.append(G - t * k + (k if run.delay else 0))
    return out


@pytest.mark.parametrize("cfg", [0, 2, 4])
def test_active_set_sizes_match_closed_form_on_the_benchmark_schedules(cfg):
    model, run, *_ = D.model_run(cfg)
    if run.batch > 2:
        run = RunShape(**{**run.__dict__, "batch": 2})
    acts, commits, _ = simulate_schedule(run, seed=cfg)
    want = _closed_form_sizes(run)
    for t in range(run.steps):
        for b in range(run.batch):
            assert len(acts[t][b]) == want[t]
            assert acts[t][b] == sorted(set(acts[t][b]))


def test_greedy_sizes_are_bounded_and_contain_the_order():
    model, run, _, _, oseed = D.model_run(3)
    run = RunShape(**{**run.__dict__, "batch": 2})
    order = D.random_block_order(run, oseed)
    acts, commits, _ = simulate_schedule(run, order=order)
    k, w = run.k_per_step, run.window
    for t in range(run.steps):
        for b in range(run.batch):
            if t % run.refresh_interval == 0:
                assert len(acts[t][b]) == run.seq_len
            else:
                assert 1 <= len(acts[t][b]) <= 2 * k + k * (w + 1)
                assert order[b, t] in acts[t][b] and order[b, t - 1] in acts[t][b]
            assert commits[t][b] == [order[b, t]]
    # the order visits every generated position once, block by block
    for b in range(run.batch):
        assert sorted(order[b].tolist()) == list(range(run.prompt_len, run.seq_len))
        for j in range(run.n_blocks):
            blk = order[b, j * run.block_len:(j + 1) * run.block_len]
            assert blk.min() == run.prompt_len + j * run.block_len
            assert blk.max() == run.prompt_len + (j + 1) * run.block_len - 1


def _expected_stamp(run, t, p, commit_step):
    """Last step <= t at which position p was recomputed, derived from the definition of the
    variants (not from select_active): s = step that committed p (None if still masked)."""
    N, P = run.refresh_interval, run.prompt_len
    last_refresh = (t // N) * N
    if run.variant == DECODE:
        if p < P:
            return last_refresh
        if commit_step is None or commit_step >= t:
            return t                                   # still masked in the input of step t
        s = commit_step
        return max(min(s + 1, t) if run.delay else s, last_refresh)
    if run.variant == PD:
        if p < P:
            return 0
        if commit_step is None or commit_step >= t:
            return t
        s = commit_step
        return max(min(s + 1, t) if run.delay else s, last_refresh)
    if run.variant == PREFILL:
        return 0 if p < P else t
    raise AssertionError


@pytest.mark.parametrize("variant,delay", [(DECODE, 1), (DECODE, 0), (PD, 1), (PREFILL, 1)])
def test_stamps_hold_exactly_the_rows_the_schedule_implies(variant, delay):
    run = RunShape(batch=2, prompt_len=6, gen_len=24, steps=24, block_len=8, refresh_interval=5,
                   variant=variant, delay=delay)
    acts, commits, stamps = simulate_schedule(run, seed=11)
    for b in range(run.batch):
        commit_step = {}
        for t in range(run.steps):
            for p in commits[t][b]:
                commit_step[p] = t
        for t in range(run.steps):
            for p in range(run.seq_len):
                assert stamps[t][b, p] == _expected_stamp(run, t, p, commit_step.get(p)), (t, p)


def test_cached_set_is_nested_between_refreshes():
    run = RunShape(batch=1, prompt_len=6, gen_len=24, steps=24, block_len=8, refresh_interval=6)
    acts, _, _ = simulate_schedule(run, seed=5)
    L = set(range(run.seq_len))
    for t in range(1, run.steps - 1):
        if S.is_refresh_step(run, t) or S.is_refresh_step(run, t + 1):
            continue
        assert (L - set(acts[t][0])) <= (L - set(acts[t + 1][0]))


@pytest.mark.parametrize("cfg,want", [(0, 0.643), (2, 0.655), (4, 0.788)])
def test_cache_ratio_of_the_benchmark_schedules(cfg, want):
    model, run, *_ = D.model_run(cfg)
    sizes = _closed_form_sizes(run)
    assert abs(S.cache_ratio(sizes, run.seq_len) - want) < 5e-4
    # hand-expanded for the tiny configuration: L=64, refresh at 0,8,16,24, otherwise 33-t rows
    if cfg == 0:
        by_hand = sum((64 - (64 if t % 8 == 0 else 33 - t)) / 64 for t in range(32)) / 32
        assert math.isclose(S.cache_ratio(sizes, 64), by_hand, rel_tol=1e-12)
        assert math.isclose(by_hand, 1316 / 64 / 32, rel_tol=1e-12)
