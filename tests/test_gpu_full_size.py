"""GPU parity at the benchmark configurations' full widths, in the launch configuration bench.py uses.

The oracle cannot run a whole 7-8B schedule, so each configuration is checked on what it can compute:
teacher-forced leading steps (a refresh step and cached steps) element by element, and over the whole
free-running schedule the index work (active sets, candidates, stamps, commit log) against properties
that follow from the definitions of the variants at any size.
"""
import numpy as np
import pytest

import dkv_inputs as D
from dkv_inputs.configs import RunShape, DECODE, PD, GREEDY
from gpu_parity import run_side_by_side

pytestmark = pytest.mark.gpu


def test_config2_llada_shape_full_depth_leading_steps():
    # 32 layers x 4096: step 0 recomputes 512 rows (refresh), step 1 the 257 rows of Eq. 4
    model, run, ws, ps, _ = D.model_run(2)
    _, _, worst = run_side_by_side(model, run, ws, ps, steps=2)
    print("configs[2] full depth, worst relative errors:", worst)


def test_config3_greedy_long_sequence_two_layer_slice():
    # batch 4 x 1536 positions, window 4, refresh every 4 steps: steps 0..5 cover two refreshes (6144 rows)
    # and the 5-7 row Greedy steps in between
    model, run, ws, ps, oseed = D.model_run(3)
    _, _, worst = run_side_by_side(model.with_layers(2), run, ws, ps, order_seed=oseed, steps=6)
    print("configs[3] 2-layer slice, worst relative errors:", worst)


def test_config4_dream_shape_gqa_pd_two_layer_slice():
    # batch 16, 28 query heads over 4 K/V heads, prompt cached at step 0: 12288 rows, then 16 x 256
    model, run, ws, ps, _ = D.model_run(4)
    _, _, worst = run_side_by_side(model.with_layers(2), run, ws, ps, steps=2)
    print("configs[4] 2-layer slice, worst relative errors:", worst)


def _expected_active(run, t, masked, d_prev):
    """Active positions of one sequence from the definitions (Decode / PD), independent of the library."""
    L, P = run.seq_len, run.prompt_len
    if t == 0:
        return np.arange(L)
    if t % run.refresh_interval == 0:
        return np.arange(P, L) if run.variant == PD else np.arange(L)
    act = masked.copy()
    act[d_prev] = True
    return np.nonzero(act)[0]


@pytest.mark.parametrize("cfg,layers", [(2, 32), (4, 1)])
def test_whole_schedule_index_work_free_running(cfg, layers):
    """The complete schedule, free-running on the device with full-width weights: every step's active
    set, candidate set and commit must follow from the mask state the device itself produced."""
    import paper_2505_15781_amd as P
    from paper_2505_15781_amd import binding
    model, run, ws, ps, _ = D.model_run(cfg)
    model = model.with_layers(layers)
    w = binding.random_weights(model, ws)
    g = P.DkvRun(model, run, w, D.prompt_tokens(model, run, ps))
    B, L, k = run.batch, run.seq_len, run.k_per_step
    masked = np.zeros((B, L), dtype=bool)
    masked[:, run.prompt_len:] = True
    stamp = np.full((B, L), -1, dtype=np.int32)
    d_prev = [np.zeros(0, dtype=np.int64) for _ in range(B)]
    check_steps = set(range(0, 20)) | set(range(run.steps - 12, run.steps)) | set(range(0, run.steps, 7))
    for t in range(run.steps):
        ub = g.select_active(t)
        if t in check_steps:
            pos, off = g.read_rows()
            assert ub == off[-1], f"step {t}: host bound {ub} != {off[-1]} rows (exact for this variant)"
        g.denoise_step(t)
        dpos = g.decoded_pos[t].cpu().numpy()
        if t in check_steps:
            cpos, ctok, cconf, coff = g.read_candidates()
        lo = run.prompt_len + (t // run.steps_per_block) * run.block_len
        for b in range(B):
            want = _expected_active(run, t, masked[b], d_prev[b])
            stamp[b, want] = t
            if t in check_steps:
                assert np.array_equal(pos[off[b]:off[b + 1]], want), f"step {t} seq {b}: active set"
                cand = want[masked[b, want] & (want >= lo) & (want < lo + run.block_len)]
                assert np.array_equal(cpos[coff[b]:coff[b + 1]], cand), f"step {t} seq {b}: candidates"
                # the commit is the most confident candidate, lowest position on ties
                conf = cconf[coff[b]:coff[b + 1]]
                order = np.lexsort((cand, -conf.astype(np.float64)))
                assert np.array_equal(dpos[b], cand[order[:k]]), f"step {t} seq {b}: commit"
                toks = ctok[coff[b]:coff[b + 1]]
                assert np.array_equal(g.decoded_tok[t, b].cpu().numpy(), toks[order[:k]])
                assert (toks != model.mask_id).all() and (conf > 0).all() and (conf <= 1).all()
            assert masked[b, dpos[b]].all(), f"step {t}: committed an unmasked position"
            masked[b, dpos[b]] = False
            d_prev[b] = dpos[b].astype(np.int64)
    assert not masked.any()
    assert np.array_equal(g.masked.cpu().numpy().astype(bool), masked)
    assert np.array_equal(g.stamp.cpu().numpy(), stamp)
    toks = g.tokens.cpu().numpy()
    assert (toks[:, run.prompt_len:] != model.mask_id).all()
    g.close()
