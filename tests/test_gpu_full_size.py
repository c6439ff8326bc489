"""GPU parity at the benchmark configurations' full widths, in the launch configuration bench.py uses.

The oracle cannot run a whole 7-8B schedule, so each configuration is checked on what it can compute, always
at the flat bars (1e-2 relative with bf16 storage). At full width one block of bf16-operand arithmetic is
already at 0.6-0.8e-2 against a float64 oracle that rounds nothing (the operand roundings alone, simulated on
the CPU, give 0.85e-2), so beyond the leading steps the bar is applied block by block, where Algorithm 1
defines the computation, and the end-to-end drift of a stack of blocks is recorded but not asserted:
  * every layer on its own at full depth: the device's own input rows of a layer and that layer's cache
    go through the oracle's one-block arithmetic (Algorithm 1 lines 3-6; Eq. 4) at steps from the whole
    schedule (first refresh, first cached step, a later refresh, the cached step after it, the middle, the
    last step);
  * whole teacher-forced schedules on 2-layer slices of the full width, with schedules shortened so that the
    oracle finishes: every row regime (2 ... 512 rows), refreshes and the cached steps after them,
    Greedy steps in several blocks, PD refreshes of the generated region. Every block and the head of every
    step are held to the bar on the device's own inputs; index state, commits and cache positions are
    compared end to end; the end-to-end float errors are printed;
  * the leading steps of the real schedules (the large launches: 6144 and 12288 rows);
  * over the whole free-running schedule the index work (active sets, candidates, stamps, commit log)
    against the oracle's schedule functions fed with the device's own mask state.
"""
import numpy as np
import pytest
import torch

import dkv_inputs as D
from dkv_inputs.configs import RunShape, DECODE, PD, GREEDY, RANDOM_ORDER, CENTER_CUR
from gpu_parity import run_side_by_side, check_close, tolerances
from oracle import model as OM
from oracle import schedule as S

pytestmark = pytest.mark.gpu


def test_config2_full_depth_every_checked_layer_alone_and_recorded_end_to_end_drift():
    """configs[2] at its 32 layers. Steps 0-1 run side by side with the oracle end to end: index work is
    asserted, the end-to-end float drift of the 32-layer bf16 stack is only printed (it is a figure of the
    arithmetic type, recorded in the design notes, not a bar). The bar is applied where the method is defined,
    per block: at steps 0, 1, 8, 9, 128 and 255 of the free-running generation the input rows the device fed
    to a layer, and the layer's cache as the device holds it, are pushed through the oracle's block and
    compared with the rows the device handed to the next layer and with the K/V rows it stored."""
    import paper_2505_15781_amd as P
    from paper_2505_15781_amd import binding
    model, run, ws, ps, _ = D.model_run(2)
    tol = tolerances(model.dtype)
    synth = D.SynthWeights(model, ws)
    w_dev = binding.upload_weights(model, synth)
    g, st, worst = run_side_by_side(model, run, ws, ps, steps=2, float_asserts=False, synth=synth, w_dev=w_dev)
    print("configs[2] full depth, end-to-end relative errors after 32 layers (recorded, not a bar):", worst, flush=True)
    g.close()
    del g, st
    torch.cuda.empty_cache()

    g = P.DkvRun(model, run, w_dev, D.prompt_tokens(model, run, ps))
    g.capture_hidden()
    check_steps = {0: (0, 1, 15, 31), 1: (0, 1, 15, 31), 8: (0, 16, 31), 9: (0, 16, 31), 128: (0, 16, 31),
                   255: (0, 16, 31)}
    worst_layer = 0.0
    for t in range(run.steps):
        g.denoise_step(t)
        if t not in check_steps:
            continue
        pos, off = g.read_rows()
        for l in check_steps[t]:
            h_in = g.read_hidden(l).astype(np.float64)
            h_out = g.read_hidden(l + 1)
            K = g.k_cache[l].float().cpu().numpy().astype(np.float64)
            V = g.v_cache[l].float().cpu().numpy().astype(np.float64)
            K_dev, V_dev = K.copy(), V.copy()
            ref = OM.layer_forward(model, synth.layer(l), h_in, pos.astype(np.int64), off.astype(int), K, V)
            l2, mx = check_close(h_out, ref, tol, f"step {t} layer {l} output rows")
            worst_layer = max(worst_layer, l2, mx)
            for b in range(run.batch):
                p = pos[off[b]:off[b + 1]]
                check_close(K_dev[b][:, p], K[b][:, p], tol, f"step {t} layer {l} stored K rows")
                check_close(V_dev[b][:, p], V[b][:, p], tol, f"step {t} layer {l} stored V rows")
            print(f"step {t} ({len(pos)} rows) layer {l}: rel L2 {l2:.2e} max {mx:.2e}", flush=True)
    print("configs[2] full depth, worst single-layer relative error:", worst_layer, flush=True)
    g.close()


def test_llada_width_two_layers_whole_schedule_every_row_regime():
    """The configs[2] sequence (256 + 256 positions, blocks of 32, refresh every 8 steps) on a 2-layer slice
    of the full width, whole schedule, with 8 commits per step so that the oracle finishes: 512 rows at the
    four refreshes and 256, 248, ... 16 rows in between, i.e. every tile shape and option the projections of a
    real generation use at the model's own N and K (one and two rows of tiles, split K on the output and down
    projections, streamed weights, fused SwiGLU), each refresh followed by cached steps."""
    model, _, ws, ps, _ = D.model_run(2)
    run = RunShape(batch=1, prompt_len=256, gen_len=256, steps=32, block_len=32, refresh_interval=8, variant=DECODE)
    _, _, worst = run_side_by_side(model.with_layers(2), run, ws, ps, per_block=True, float_asserts=False)
    print("LLaDA width, 2 layers, 32-step schedule, worst relative errors:", worst, flush=True)


def test_llada_width_two_layers_one_commit_per_step_down_to_two_rows():
    """One commit per step as in configs[2], on a shorter sequence: 128 rows at the refreshes, 64 ... 2 rows in
    between (the single-row-of-tiles launches), run as a generation does: without the debug copy of the logits,
    so the tokens and confidences are what the head is compared on."""
    model, _, ws, ps, _ = D.model_run(2)
    run = RunShape(batch=1, prompt_len=64, gen_len=64, steps=64, block_len=32, refresh_interval=8, variant=DECODE)
    _, _, worst = run_side_by_side(model.with_layers(2), run, ws, ps, with_logits=False, per_block=True, float_asserts=False)
    print("LLaDA width, 2 layers, 64 single-commit steps, worst relative errors:", worst, flush=True)


def test_config3_greedy_long_sequence_two_layer_slice():
    # batch 4 x 1536 positions, window 4, refresh every 4 steps: steps 0..5 cover two refreshes (6144 rows)
    # and the 5-7 row Greedy steps in between
    model, run, ws, ps, oseed = D.model_run(3)
    _, _, worst = run_side_by_side(model.with_layers(2), run, ws, ps, order_seed=oseed, steps=6)
    print("configs[3] 2-layer slice, worst relative errors:", worst, flush=True)


def test_llada_width_two_layers_greedy_whole_schedule_over_four_blocks():
    """The Greedy variant of configs[3] (window 4, refresh every 4 steps, predefined order) on a shorter
    sequence (2 x 256 positions), whole schedule: Greedy steps in every block, windows clipped at block and
    sequence ends, the previous step's commit across block boundaries, a refresh every fourth step."""
    model, _, ws, ps, oseed = D.model_run(3)
    run = RunShape(batch=2, prompt_len=224, gen_len=32, steps=32, block_len=8, refresh_interval=4, variant=GREEDY,
                   window=4, window_center=CENTER_CUR, include_prev=1, remask=RANDOM_ORDER)
    _, _, worst = run_side_by_side(model.with_layers(2), run, ws, ps, order_seed=oseed, per_block=True, float_asserts=False)
    print("LLaDA width, 2 layers, Greedy 32-step schedule, worst relative errors:", worst, flush=True)


def test_config4_dream_shape_gqa_pd_two_layer_slice():
    # batch 16, 28 query heads over 4 K/V heads, prompt cached at step 0: 12288 rows, then 16 x 256
    model, run, ws, ps, _ = D.model_run(4)
    _, _, worst = run_side_by_side(model.with_layers(2), run, ws, ps, steps=2)
    print("configs[4] 2-layer slice, worst relative errors:", worst, flush=True)


def test_dream_width_two_layers_pd_whole_schedule_with_refreshes():
    """The PD variant of configs[4] (batch 16, grouped K/V heads, prompt cached once, the generated region
    refreshed every 4 steps) on a shorter sequence, whole schedule: 1024 rows at step 0, 512 at the refreshes,
    16 x (33 - t) rows on the cached steps after them."""
    model, _, ws, ps, _ = D.model_run(4)
    run = RunShape(batch=16, prompt_len=32, gen_len=32, steps=32, block_len=8, refresh_interval=4, variant=PD)
    _, _, worst = run_side_by_side(model.with_layers(2), run, ws, ps, per_block=True, float_asserts=False)
    print("Dream width, 2 layers, PD 32-step schedule, worst relative errors:", worst, flush=True)


@pytest.mark.parametrize("cfg,layers", [(2, 32), (3, 1), (4, 1)])
def test_whole_schedule_index_work_free_running(cfg, layers):
    """The complete schedule, free-running on the device with full-width weights: every step's active
    set and candidate set must be what the oracle's schedule functions give for the mask state the device
    itself produced, and the commit must follow from the device's confidences (or the predefined order)."""
    import paper_2505_15781_amd as P
    from paper_2505_15781_amd import binding
    model, run, ws, ps, oseed = D.model_run(cfg)
    model = model.with_layers(layers)
    w = binding.random_weights(model, ws)
    order = D.random_block_order(run, oseed) if run.remask == RANDOM_ORDER else None
    g = P.DkvRun(model, run, w, D.prompt_tokens(model, run, ps), order=order)
    B, L, k = run.batch, run.seq_len, run.k_per_step
    masked = np.zeros((B, L), dtype=bool)
    masked[:, run.prompt_len:] = True
    stamp = np.full((B, L), -1, dtype=np.int32)
    d_prev = [[] for _ in range(B)]
    exact_bound = run.variant != GREEDY
    check_steps = set(range(0, 20)) | set(range(run.steps - 12, run.steps)) | set(range(0, run.steps, 7))
    if run.variant == GREEDY:       # every step: the sets are a few rows, and block ends are where windows clip
        check_steps = set(range(run.steps))
    for t in range(run.steps):
        ub = g.select_active(t)
        if t in check_steps:
            pos, off = g.read_rows()
            assert ub == off[-1] if exact_bound else ub >= off[-1], f"step {t}: host bound {ub}, {off[-1]} rows"
        g.denoise_step(t)
        dpos = g.decoded_pos[t].cpu().numpy()
        if t in check_steps:
            cpos, ctok, cconf, coff = g.read_candidates()
        for b in range(B):
            d_cur = None if order is None else [int(p) for p in order[b, t * k:(t + 1) * k]]
            want = np.asarray(S.select_active(run, t, masked[b], d_prev[b], d_cur), dtype=np.int64)
            stamp[b, want] = t
            if t in check_steps:
                assert np.array_equal(pos[off[b]:off[b + 1]], want), f"step {t} seq {b}: active set"
                cand = np.asarray(S.candidates(run, t, list(want), masked[b]), dtype=np.int64)
                assert np.array_equal(cpos[coff[b]:coff[b + 1]], cand), f"step {t} seq {b}: candidates"
                conf = cconf[coff[b]:coff[b + 1]]
                toks = ctok[coff[b]:coff[b + 1]]
                if order is None:
                    # the commit is the most confident candidate, lowest position on ties
                    pick = np.lexsort((cand, -conf.astype(np.float64)))[:k]
                else:
                    pick = np.asarray([int(np.nonzero(cand == p)[0][0]) for p in d_cur])
                assert np.array_equal(dpos[b], cand[pick]), f"step {t} seq {b}: commit"
                assert np.array_equal(g.decoded_tok[t, b].cpu().numpy(), toks[pick])
                assert (toks != model.mask_id).all() and (conf > 0).all() and (conf <= 1).all()
            assert masked[b, dpos[b]].all(), f"step {t}: committed an unmasked position"
            masked[b, dpos[b]] = False
            d_prev[b] = [int(p) for p in dpos[b]]
    assert not masked.any()
    assert np.array_equal(g.masked.cpu().numpy().astype(bool), masked)
    assert np.array_equal(g.stamp.cpu().numpy(), stamp)
    toks = g.tokens.cpu().numpy()
    assert (toks[:, run.prompt_len:] != model.mask_id).all()
    g.close()
