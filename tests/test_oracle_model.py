"""Pins of the oracle's arithmetic: textbook properties, special cases that must be exact,
an independent scalar-loop reconstruction, and the second (concat/reorder) formulation."""
import math
import numpy as np
import pytest
import dkv_inputs as D
from dkv_inputs.configs import (ModelShape, RunShape, FP32, DECODE, GREEDY, PD, PREFILL,
                                RANDOM_ORDER, CONFIDENCE)
from oracle import model as M, sampler as SA, schedule as S, brute, concat_reorder, attn_update
from helpers import SMALL


def _weights(model, seed=7):
    return D.SynthWeights(model, seed)


# ---------------------------------------------------------------- textbook pieces

def test_softmax_rows_sum_to_one_and_are_shift_invariant():
    rng = np.random.default_rng(0)
    s = rng.normal(size=(5, 9)) * 10
    p = M.softmax(s)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-14)
    assert np.allclose(p, M.softmax(s + 123.0), atol=1e-14)
    assert np.allclose(M.softmax(np.log(np.array([[1.0, 2.0, 5.0]]))), [[0.125, 0.25, 0.625]])


def test_rmsnorm_closed_forms():
    x = np.array([[3.0, -4.0]])                      # mean square 12.5
    assert np.allclose(M.rmsnorm(x, [1.0, 1.0], 0.0), x / math.sqrt(12.5))
    assert np.allclose(M.rmsnorm(x, [2.0, 0.5], 0.0), x / math.sqrt(12.5) * [2.0, 0.5])
    assert np.allclose(M.rmsnorm(x, [1.0, 1.0], 3.5), x / 4.0)          # eps inside the root
    y = M.rmsnorm(np.random.default_rng(1).normal(size=(4, 64)), np.ones(64), 0.0)
    assert np.allclose(np.mean(y * y, -1), 1.0)


def test_silu_values():
    assert M.silu(np.array(0.0)) == 0.0
    assert math.isclose(float(M.silu(np.array(1.0))), 1.0 / (1.0 + math.exp(-1.0)))
    assert math.isclose(float(M.silu(np.array(-2.0))), -2.0 / (1.0 + math.exp(2.0)))


def test_rope_is_a_rotation_by_position_times_frequency():
    # dh = 2: a single pair rotated by angle = pos (frequency theta^0 = 1), counter-clockwise
    x = np.array([[[1.0, 0.0]]])
    assert np.allclose(M.rope(x, [0], 10000.0), x)
    assert np.allclose(M.rope(x, [1], 10000.0), [[[math.cos(1.0), math.sin(1.0)]]])
    y = np.array([[[0.0, 1.0]]])
    assert np.allclose(M.rope(y, [2], 10000.0), [[[-math.sin(2.0), math.cos(2.0)]]])
    # dh = 4: pairs are (0,2) and (1,3); the second pair turns at theta^(-2/4)
    z = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    f = 100.0 ** (-0.5)
    assert np.allclose(M.rope(z, [3], 100.0), [[[math.cos(3.0), math.cos(3 * f), math.sin(3.0), math.sin(3 * f)]]])


def test_rope_keeps_norms_and_makes_scores_depend_on_relative_position():
    rng = np.random.default_rng(2)
    q = rng.normal(size=(1, 1, 16)); k = rng.normal(size=(1, 1, 16))
    assert np.allclose(np.linalg.norm(M.rope(q, [37], 1e4)), np.linalg.norm(q))
    a = (M.rope(q, [5], 1e4) * M.rope(k, [2], 1e4)).sum()
    b = (M.rope(q, [105], 1e4) * M.rope(k, [102], 1e4)).sum()
    c = (M.rope(q, [5], 1e4) * M.rope(k, [3], 1e4)).sum()
    assert math.isclose(a, b, rel_tol=1e-9) and not math.isclose(a, c, rel_tol=1e-3)


def test_attention_special_cases():
    rng = np.random.default_rng(3)
    q = rng.normal(size=(3, 4, 8))
    V = rng.normal(size=(2, 6, 8))
    K_equal = np.repeat(rng.normal(size=(2, 1, 8)), 6, axis=1)
    out = M.attention(q, K_equal, V, 2)                 # equal keys -> uniform weights -> mean of V
    for h in range(4):
        assert np.allclose(out[:, h], V[h // 2].mean(0))
    # a key aligned with the query and far larger than the rest picks out its own value row
    K = np.zeros((2, 6, 8)); K[:, 4, :] = 1000.0 * np.sign(q[0, 0])
    out = M.attention(q[:1, :1], K[:1], V[:1], 1)
    assert np.allclose(out[0, 0], V[0, 4], atol=1e-9)


def test_attention_matches_explicit_loops_and_gqa_is_head_sharing():
    rng = np.random.default_rng(4)
    n, Hq, Hkv, L, dh = 3, 4, 2, 5, 6
    q = rng.normal(size=(n, Hq, dh)); K = rng.normal(size=(Hkv, L, dh)); V = rng.normal(size=(Hkv, L, dh))
    out = M.attention(q, K, V, Hq // Hkv)
    for i in range(n):
        for h in range(Hq):
            kv = h // (Hq // Hkv)
            sc = [sum(q[i, h, c] * K[kv, j, c] for c in range(dh)) / math.sqrt(dh) for j in range(L)]
            e = [math.exp(s - max(sc)) for s in sc]
            for c in range(dh):
                want = sum(e[j] / sum(e) * V[kv, j, c] for j in range(L))
                assert math.isclose(out[i, h, c], want, rel_tol=1e-11, abs_tol=1e-13)
    rep = M.attention(q, np.repeat(K, 2, axis=0), np.repeat(V, 2, axis=0), 1)
    assert np.allclose(out, rep, atol=1e-14)


def test_predict_excludes_mask_breaks_ties_low_and_reports_softmax_max():
    lg = np.array([[0.0, 2.0, 2.0, 9.0], [1.0, 0.5, 0.25, 100.0]])
    tok, conf = SA.predict(lg, mask_id=3)
    assert tok.tolist() == [1, 0]
    assert math.isclose(conf[0], math.exp(2) / (1 + 2 * math.exp(2)), rel_tol=1e-6)
    assert math.isclose(conf[1], math.exp(1) / (math.exp(1) + math.exp(0.5) + math.exp(0.25)), rel_tol=1e-6)
    assert conf.dtype == np.float32
    with pytest.raises(FloatingPointError):
        SA.predict(np.array([[0.0, np.nan, 1.0]]), 2)


def test_top_k_prefers_confidence_then_lower_position():
    assert SA.top_k_positions([5, 7, 9, 11], np.float32([0.2, 0.9, 0.9, 0.1]), 2) == [7, 9]
    assert SA.top_k_positions([5, 7, 9, 11], np.float32([0.2, 0.9, 0.9, 0.1]), 3) == [7, 9, 5]
    assert SA.top_k_positions([5, 7], np.float32([0.5, 0.5]), 1) == [5]


# ---------------------------------------------------------------- exact special cases of the method

def _prompt(model, run, seed=9):
    return D.prompt_tokens(model, run, seed)


def _logits_by_pos(log, b):
    return {p: log.cand_logits[b][i] for i, p in enumerate(log.cand[b])}


def test_refresh_every_step_equals_cache_free_recomputation():
    model = SMALL
    run = RunShape(batch=2, prompt_len=5, gen_len=8, steps=8, block_len=4, refresh_interval=1)
    w, prompt = _weights(model), _prompt(model, run)
    st = SA.init_state(model, run, prompt)
    for t in range(run.steps):
        tokens_in = st.tokens.copy()
        log = SA.denoise_step(model, w, run, st, t, keep_logits=True, keep_hidden=True)
        h_full, store_full = M.full_forward(model, w, tokens_in)
        assert all(a == list(range(run.seq_len)) for a in log.active)
        assert np.array_equal(log.hidden, h_full)                      # same arithmetic, bit for bit
        assert np.array_equal(st.store.K, store_full.K) and np.array_equal(st.store.V, store_full.V)
        lg_full = M.logits_of(model, w, h_full).reshape(run.batch, run.seq_len, -1)
        for b in range(run.batch):
            for p, lg in _logits_by_pos(log, b).items():
                assert np.allclose(lg, lg_full[b, p], rtol=1e-13, atol=1e-15)   # BLAS blocking varies with row count


def _run_collect(model, w, run, prompt, order=None, forced=None):
    st = SA.generate(model, w, run, prompt, order=order, forced=forced, keep_logits=True)
    return st


@pytest.mark.parametrize("N", [2, 3, 100])
def test_one_layer_model_with_one_step_delay_reproduces_full_recomputation(N):
    # With one layer K/V of a position depend on its own token only, so rows cached one step
    # after decoding equal the recomputed ones and Decode is exact; without the delay the row
    # was computed from MASK and must differ.
    model = ModelShape(**{**SMALL.__dict__, "n_layers": 1})
    base = dict(batch=2, prompt_len=5, gen_len=8, steps=8, block_len=4)
    w = _weights(model)
    prompt = _prompt(model, RunShape(refresh_interval=1, **base))
    ref = _run_collect(model, w, RunShape(refresh_interval=1, **base), prompt)
    forced = [(l.pos, l.tok) for l in ref.logs]
    got = _run_collect(model, w, RunShape(refresh_interval=N, **base), prompt)
    for lr, lg in zip(ref.logs, got.logs):
        assert np.array_equal(lr.pos, lg.pos) and np.array_equal(lr.tok, lg.tok)
        for b in range(2):
            assert lr.cand[b] == lg.cand[b]
            assert np.allclose(lr.cand_logits[b], lg.cand_logits[b], rtol=1e-11, atol=1e-13)
    nodelay = _run_collect(model, w, RunShape(refresh_interval=N, delay=0, **base), prompt, forced=forced)
    diffs = [np.max(np.abs(lr.cand_logits[0] - ln.cand_logits[0])) for lr, ln in zip(ref.logs, nodelay.logs)
             if lr.t % N != 0 and lr.t >= 2]
    assert max(diffs) > 1e-6


@pytest.mark.parametrize("N,variant", [(1, DECODE), (3, DECODE), (100, DECODE), (2, PD), (2, PREFILL)])
def test_shifted_logits_read_the_previous_row_and_stay_exact_with_one_layer(N, variant):
    # Appendix B (Un-Shift): the prediction for position q is the output of row q - 1. Checked against a
    # cache-free forward over all positions read at q - 1; with one layer the cached run must agree exactly
    # for any refresh interval, and it must differ from reading the logits at q itself.
    model = ModelShape(**{**SMALL.__dict__, "n_layers": 1})
    run = RunShape(batch=2, prompt_len=5, gen_len=8, steps=8, block_len=4, refresh_interval=N, variant=variant,
                   shift_logits=1)
    w, prompt = _weights(model), _prompt(model, run)
    st = SA.init_state(model, run, prompt)
    differs = False
    for t in range(run.steps):
        tokens_in = st.tokens.copy()
        log = SA.denoise_step(model, w, run, st, t, keep_logits=True)
        h_full, _ = M.full_forward(model, w, tokens_in)
        lg_full = M.logits_of(model, w, h_full).reshape(run.batch, run.seq_len, -1)
        for b in range(run.batch):
            assert all(q - 1 in log.active[b] for q in log.cand[b])
            for q, lg in _logits_by_pos(log, b).items():
                assert np.allclose(lg, lg_full[b, q - 1], rtol=1e-11, atol=1e-13)
                differs |= np.max(np.abs(lg - lg_full[b, q])) > 1e-6
    assert differs


def test_shifted_logits_with_refresh_every_step_equal_cache_free_recomputation_at_depth():
    model = SMALL
    run = RunShape(batch=2, prompt_len=5, gen_len=8, steps=8, block_len=4, refresh_interval=1, shift_logits=1)
    w, prompt = _weights(model), _prompt(model, run)
    st = SA.init_state(model, run, prompt)
    for t in range(run.steps):
        tokens_in = st.tokens.copy()
        log = SA.denoise_step(model, w, run, st, t, keep_logits=True)
        h_full, _ = M.full_forward(model, w, tokens_in)
        lg_full = M.logits_of(model, w, h_full).reshape(run.batch, run.seq_len, -1)
        for b in range(run.batch):
            for q, lg in _logits_by_pos(log, b).items():
                assert np.allclose(lg, lg_full[b, q - 1], rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("include_prev", [1, 0])
def test_one_layer_greedy_is_exact_only_when_the_previous_commit_is_recomputed(include_prev):
    model = ModelShape(**{**SMALL.__dict__, "n_layers": 1})
    base = dict(batch=1, prompt_len=5, gen_len=8, steps=8, block_len=4, remask=RANDOM_ORDER)
    order = D.random_block_order(RunShape(refresh_interval=1, **base), 21)
    w = _weights(model)
    prompt = _prompt(model, RunShape(refresh_interval=1, **base))
    ref = _run_collect(model, w, RunShape(refresh_interval=1, **base), prompt, order=order)
    forced = [(l.pos, l.tok) for l in ref.logs]
    run = RunShape(refresh_interval=100, variant=GREEDY, window=2, include_prev=include_prev, **base)
    got = _run_collect(model, w, run, prompt, order=order, forced=forced)
    worst = 0.0
    for lr, lg in zip(ref.logs, got.logs):
        ref_l = _logits_by_pos(lr, 0)
        for p, row in _logits_by_pos(lg, 0).items():
            worst = max(worst, float(np.max(np.abs(row - ref_l[p]))))
    assert (worst < 1e-11) if include_prev else (worst > 1e-6)


def test_layer0_cache_rows_always_equal_recomputed_layer0_rows():
    model = SMALL
    run = RunShape(batch=1, prompt_len=5, gen_len=8, steps=8, block_len=8, refresh_interval=4)
    w, prompt = _weights(model), _prompt(model, run)
    st = SA.init_state(model, run, prompt)
    for t in range(run.steps):
        SA.denoise_step(model, w, run, st, t)
        # the state now holds step t's commits as tokens, but the cache rows of those positions
        # were computed from MASK at step t: compare against the tokens fed at step t.
        fed = st.tokens.copy()
        fed[0, st.logs[-1].pos[0]] = model.mask_id
        _, full = M.full_forward(model, w, fed)
        assert np.allclose(st.store.K[0], full.K[0], rtol=1e-12, atol=1e-14)
        assert np.allclose(st.store.V[0], full.V[0], rtol=1e-12, atol=1e-14)
        assert not np.isnan(st.store.K).any()


def test_deeper_model_really_is_an_approximation_between_refreshes():
    model = SMALL
    base = dict(batch=1, prompt_len=5, gen_len=8, steps=8, block_len=8)
    w = _weights(model)
    prompt = _prompt(model, RunShape(refresh_interval=1, **base))
    ref = _run_collect(model, w, RunShape(refresh_interval=1, **base), prompt)
    forced = [(l.pos, l.tok) for l in ref.logs]
    got = _run_collect(model, w, RunShape(refresh_interval=4, **base), prompt, forced=forced)
    d = [float(np.max(np.abs(a.cand_logits[0] - b.cand_logits[0]))) for a, b in zip(ref.logs, got.logs)]
    # refresh steps are exact; in between, deeper-layer rows of cached positions are stale
    assert d[0] == 0.0 and d[4] == 0.0
    assert all(1e-9 < x < 1.0 for i, x in enumerate(d) if i % 4)


def test_head_on_candidates_equals_head_on_all_active_rows_restricted():
    model = SMALL
    run = RunShape(batch=2, prompt_len=5, gen_len=8, steps=8, block_len=4, refresh_interval=3)
    w, prompt = _weights(model), _prompt(model, run)
    a, b = SA.init_state(model, run, prompt), SA.init_state(model, run, prompt)
    for t in range(run.steps):
        la = SA.denoise_step(model, w, run, a, t, keep_logits=True)
        lb = SA.denoise_step(model, w, run, b, t, keep_logits=True, head_all_rows=True)
        for s in range(2):
            assert np.allclose(la.cand_logits[s], lb.cand_logits[s], rtol=1e-12, atol=1e-14)
        assert np.array_equal(la.pos, lb.pos) and np.array_equal(la.tok, lb.tok)


@pytest.mark.parametrize("N", [1, 3, 100])
def test_position_indexed_store_agrees_with_concat_reorder_formulation(N):
    model = SMALL
    run = RunShape(batch=2, prompt_len=5, gen_len=8, steps=8, block_len=4, refresh_interval=N)
    w, prompt = _weights(model), _prompt(model, run)
    st = SA.generate(model, w, run, prompt, keep_logits=True)
    alt = concat_reorder.generate_decode(model, w, run, prompt)
    for b in range(run.batch):
        for t, (cand, lg, chosen, toks) in enumerate(alt[b]):
            log = st.logs[t]
            assert cand == log.cand[b]
            assert np.allclose(lg, log.cand_logits[b], rtol=1e-10, atol=1e-12)
            assert chosen == log.pos[b].tolist() and toks == log.tok[b].tolist()


@pytest.mark.parametrize("variant", [DECODE, PD, GREEDY])
def test_running_store_equals_literal_eq4_assembly_from_full_history(variant):
    model = ModelShape(n_layers=2, d_model=8, n_q_heads=2, n_kv_heads=1, head_dim=4, d_ffn=12,
                       vocab=16, mask_id=15, dtype=FP32)
    kw = dict(batch=1, prompt_len=3, gen_len=5, steps=5, block_len=5, refresh_interval=3, variant=variant)
    order = None
    if variant == GREEDY:
        kw.update(remask=RANDOM_ORDER, window=2)
        order = D.random_block_order(RunShape(**kw), 4)
    run = RunShape(**kw)
    w, prompt = _weights(model, 3), _prompt(model, run, 5)
    st = SA.init_state(model, run, prompt)
    hist_k, hist_v, active_hist = [], [], []
    for t in range(run.steps):
        tokens_in = st.tokens[0].tolist()
        log = SA.denoise_step(model, w, run, st, t, order=order, keep_logits=True)
        active_hist.append(log.active[0])
        lg = brute.step_logits(model, w, tokens_in, active_hist, hist_k, hist_v, t)
        for i, p in enumerate(log.cand[0]):
            assert np.allclose(log.cand_logits[0][i], lg[p], rtol=1e-10, atol=1e-12)


def test_attn_update_scatters_then_attends_over_everything():
    shape = D.AttnUpdateShape(batch=2, n_q_heads=4, n_kv_heads=2, seq_len=9, head_dim=4, dtype=FP32)
    c = D.attn_update_case(shape, 3, 77)
    kc, vc = c["k_cache"].astype(np.float64), c["v_cache"].astype(np.float64)
    k0 = kc.copy()
    out = attn_update.attn_update(kc, vc, c["q"], c["k_new"], c["v_new"], c["active_idx"], c["active_off"])
    for b in range(2):
        rows = range(c["active_off"][b], c["active_off"][b + 1])
        pos = c["active_idx"][c["active_off"][b]:c["active_off"][b + 1]].tolist()
        for r, p in zip(rows, pos):
            assert np.array_equal(kc[b, :, p, :], c["k_new"][r].astype(np.float64))
        untouched = [p for p in range(9) if p not in pos]
        assert np.array_equal(kc[b][:, untouched], k0[b][:, untouched])
        for r in rows:
            for h in range(4):
                s = kc[b, h // 2] @ c["q"][r, h].astype(np.float64) / 2.0
                want = M.softmax(s) @ vc[b, h // 2]
                assert np.allclose(out[r, h], want, rtol=1e-12)


def test_tiny_configuration_runs_and_respects_the_schedule():
    model, run, ws, ps, _ = D.model_run(0)
    w = D.SynthWeights(model, ws)
    st = SA.generate(model, w, run, D.prompt_tokens(model, run, ps))
    assert not st.masked.any() and (st.tokens != model.mask_id).all()
    committed = np.concatenate([l.pos[0] for l in st.logs])
    assert sorted(committed.tolist()) == list(range(32, 64))
    for l in st.logs:
        assert len(l.active[0]) == (64 if l.t % 8 == 0 else 33 - l.t)
