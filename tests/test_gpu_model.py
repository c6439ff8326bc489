"""GPU parity of whole denoising runs against the oracle: index state bit-exact, floats within
1e-2 relative (bf16 storage) or 1e-5 (fp32 mode)."""
import numpy as np
import pytest

import dkv_inputs as D
from dkv_inputs.configs import (ModelShape, RunShape, BF16, FP32, DECODE, GREEDY, PREFILL, PD, RANDOM_ORDER,
                                CENTER_PREV, SCOPE_ALL, SCOPE_GEN)
from gpu_parity import run_side_by_side

pytestmark = pytest.mark.gpu

SMALL_BF16 = ModelShape(n_layers=3, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=384,
                        vocab=520, mask_id=519, dtype=BF16)
SMALL_FP32 = ModelShape(n_layers=2, d_model=96, n_q_heads=6, n_kv_heads=2, head_dim=32, d_ffn=160,
                        vocab=300, mask_id=299, dtype=FP32)


def test_tiny_configuration_free_running_reproduces_the_oracle_tokens():
    model, run, ws, ps, _ = D.model_run(0)
    g, st, worst = run_side_by_side(model, run, ws, ps, teacher_forced=False)
    print("configs[0] worst relative errors", worst)
    assert np.array_equal(g.decoded_pos.cpu().numpy()[:, 0, 0], np.array([l.pos[0, 0] for l in st.logs]))


@pytest.mark.parametrize("model", [SMALL_BF16, SMALL_FP32], ids=["bf16", "fp32"])
@pytest.mark.parametrize("variant", [DECODE, PD, PREFILL])
def test_cache_variants_teacher_forced(model, variant):
    run = RunShape(batch=3, prompt_len=21, gen_len=24, steps=24, block_len=8, refresh_interval=5, variant=variant)
    run_side_by_side(model, run, 7, 8)


ODD_BF16 = ModelShape(n_layers=2, d_model=200, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=328,
                      vocab=520, mask_id=519, dtype=BF16)


def test_bf16_model_whose_widths_do_not_fit_the_tile_kernel_takes_the_unfused_path():
    """d_model = 200 is no multiple of the projections' K tile: register-staged projection kernel, SwiGLU and the
    vocabulary statistics in launches of their own (fp32 logits written and read back)."""
    run = RunShape(batch=2, prompt_len=13, gen_len=16, steps=16, block_len=8, refresh_interval=4)
    run_side_by_side(ODD_BF16, run, 31, 32)


def test_block_by_block_and_without_the_debug_copy_of_the_logits():
    """A small model whose widths fit the tile kernel (SwiGLU and the vocabulary statistics in the projections'
    epilogues): every block on the device's own inputs, and the head compared on tokens and confidences only, as
    in a generation, where the logits are never written."""
    run = RunShape(batch=3, prompt_len=21, gen_len=24, steps=24, block_len=8, refresh_interval=5, variant=DECODE)
    run_side_by_side(SMALL_BF16, run, 33, 34, per_block=True)
    run_side_by_side(SMALL_BF16, run, 33, 34, with_logits=False)


def test_two_commits_per_step_and_no_delay_ablation():
    run = RunShape(batch=2, prompt_len=10, gen_len=32, steps=16, block_len=16, refresh_interval=4)
    run_side_by_side(SMALL_BF16, run, 9, 10)
    run0 = RunShape(batch=2, prompt_len=10, gen_len=32, steps=16, block_len=16, refresh_interval=4, delay=0)
    run_side_by_side(SMALL_FP32, run0, 9, 10)


@pytest.mark.parametrize("center,include_prev", [(0, 1), (CENTER_PREV, 1), (0, 0)])
def test_greedy_variant_with_window(center, include_prev):
    run = RunShape(batch=2, prompt_len=9, gen_len=24, steps=24, block_len=12, refresh_interval=4, variant=GREEDY,
                   window=4, window_center=center, include_prev=include_prev, remask=RANDOM_ORDER)
    run_side_by_side(SMALL_BF16, run, 11, 12, order_seed=13)


@pytest.mark.parametrize("variant", [DECODE, PD, PREFILL, GREEDY])
def test_shifted_logits_use_the_row_before_each_candidate(variant):
    """Appendix B (Un-Shift): row q - 1 predicts position q and joins the active set; several blocks so that
    the extra rows appear in the middle of the generated region, batch 3 so that they appear at sequence starts
    of the row list."""
    kw = dict(remask=RANDOM_ORDER, window=2) if variant == GREEDY else {}
    run = RunShape(batch=3, prompt_len=11, gen_len=24, steps=24, block_len=8, refresh_interval=5, variant=variant,
                   shift_logits=1, **kw)
    run_side_by_side(SMALL_FP32, run, 21, 22, order_seed=23 if variant == GREEDY else None)
    run_side_by_side(SMALL_BF16, run, 21, 22, order_seed=23 if variant == GREEDY else None)


def test_shifted_logits_free_running_fp32_reproduces_the_oracle_tokens():
    run = RunShape(batch=2, prompt_len=9, gen_len=16, steps=16, block_len=8, refresh_interval=4, shift_logits=1)
    g, st, _ = run_side_by_side(SMALL_FP32, run, 24, 25, teacher_forced=False)
    assert np.array_equal(g.decoded_pos.cpu().numpy(), np.stack([l.pos for l in st.logs]))
    assert np.array_equal(g.decoded_tok.cpu().numpy(), np.stack([l.tok for l in st.logs]))


def test_explicit_refresh_out_of_schedule():
    run = RunShape(batch=2, prompt_len=7, gen_len=16, steps=16, block_len=16, refresh_interval=100)
    run_side_by_side(SMALL_FP32, run, 14, 15, forced_scopes={3: SCOPE_ALL, 9: SCOPE_GEN})


def test_empty_prompt_and_single_block():
    run = RunShape(batch=1, prompt_len=0, gen_len=16, steps=16, block_len=16, refresh_interval=3)
    run_side_by_side(SMALL_BF16, run, 16, 17)


def test_step_order_and_bad_descriptors_are_reported():
    import paper_2505_15781_amd as P
    from paper_2505_15781_amd import binding
    model, run, ws, ps, _ = D.model_run(0)
    synth = D.SynthWeights(model, ws)
    w = binding.upload_weights(model, synth)
    g = P.DkvRun(model, run, w, D.prompt_tokens(model, run, ps))
    with pytest.raises(P.DkvError) as e:
        g.denoise_step(1)
    assert e.value.code == -2
    with pytest.raises(P.DkvError):
        g.refresh(7)
    bad = RunShape(batch=1, prompt_len=4, gen_len=8, steps=8, block_len=3, refresh_interval=2)
    with pytest.raises(P.DkvError):
        P.DkvRun(model, bad, w, np.zeros((1, 4), dtype=np.int32))
