"""Drives the HIP library and the oracle side by side on the same seeded inputs (GPU tests only)."""
import numpy as np
import torch

import dkv_inputs as D
from dkv_inputs.configs import BF16, FP32, RANDOM_ORDER
from oracle import sampler as SA
from oracle import model as OM
from helpers import rel_err


def tolerances(dtype):
    """Relative bars of the build at any depth and width: 1e-5 in fp32 mode, 1e-2 with bf16 storage, per
    tensor, as L2-relative and as max-abs over max-abs."""
    return 1e-5 if dtype != BF16 else 1e-2


def check_close(got, ref, tol, what, enforce=True):
    l2, mx = rel_err(got, ref)
    if enforce:
        assert l2 <= tol and mx <= tol, f"{what}: rel L2 {l2:.3e}, rel max {mx:.3e} > {tol:.0e}"
    return l2, mx


def run_side_by_side(model, run, wseed, pseed, order_seed=None, teacher_forced=True, steps=None,
                     forced_scopes=None, check_hidden=True, verbose=False, float_asserts=True, with_logits=True,
                     synth=None, w_dev=None, per_block=False):
    """Steps both sides; asserts index state bit-exact and floats within tolerance.
    float_asserts=False only records the float errors (index work is still asserted): for end-to-end
    figures of deep stacks, whose layers are held to the bar one by one elsewhere.
    per_block=True additionally holds every block of every step to the bar on its own: the rows the device
    fed to layer l and the device's cache of layer l go through the oracle's block (Algorithm 1 lines 3-6),
    whose output rows and fresh K/V rows are compared with what the device handed on and stored; likewise the
    vocabulary head on the device's own final rows.
    with_logits=False runs the step as a generation does, without the debug copy of the logits; tokens and
    confidences are then the only outputs of the head that are compared.
    Returns (gpu run object, oracle state, worst relative errors)."""
    import paper_2505_15781_amd as P
    from paper_2505_15781_amd import binding
    tol = tolerances(model.dtype)
    if synth is None:
        synth = D.SynthWeights(model, wseed, hold_float64=model.n_layers <= 4)
    prompt = D.prompt_tokens(model, run, pseed)
    order = D.random_block_order(run, order_seed) if run.remask == RANDOM_ORDER else None
    if w_dev is None:
        w_dev = binding.upload_weights(model, synth)
    g = P.DkvRun(model, run, w_dev, prompt, order=order)
    st = SA.init_state(model, run, prompt)
    B, k, V = run.batch, run.k_per_step, model.vocab
    n_steps = run.steps if steps is None else steps
    worst = {"logits": 0.0, "hidden": 0.0, "conf": 0.0}
    if per_block:
        g.capture_hidden()
        worst.update({"block_out": 0.0, "block_kv": 0.0, "head_logits": 0.0, "head_conf": 0.0})
    for t in range(n_steps):
        scope = None if forced_scopes is None else forced_scopes.get(t)
        if scope is not None:
            g.refresh(scope)
        log = SA.denoise_step(model, synth, run, st, t, order=order, forced_scope=scope,
                              keep_logits=True, keep_hidden=check_hidden)
        ub = g.select_active(t)
        pos, off = g.read_rows()
        want_pos = np.concatenate([np.asarray(a, dtype=np.int32) for a in log.active])
        want_off = np.concatenate([[0], np.cumsum([len(a) for a in log.active])]).astype(np.int32)
        assert np.array_equal(off, want_off), f"step {t}: row offsets {off} != {want_off}"
        assert np.array_equal(pos, want_pos), f"step {t}: active positions differ"
        assert ub >= len(want_pos), f"step {t}: host bound {ub} below {len(want_pos)} rows"
        n_cand = sum(len(c) for c in log.cand)
        logits = None
        if with_logits:
            logits = torch.full((B * run.block_len, V), float("nan"), dtype=torch.float32, device="cuda")
        fpos = ftok = None
        if teacher_forced:
            fpos = torch.as_tensor(log.pos, dtype=torch.int32, device="cuda").contiguous()
            ftok = torch.as_tensor(log.tok, dtype=torch.int32, device="cuda").contiguous()
        g.denoise_step(t, fpos, ftok, logits)
        cpos, ctok, cconf, coff = g.read_candidates()
        want_cpos = np.concatenate([np.asarray(c, dtype=np.int32) for c in log.cand])
        assert np.array_equal(cpos, want_cpos), f"step {t}: candidate positions differ"
        ref_logits = np.concatenate(log.cand_logits, axis=0)
        if with_logits:
            got_logits = logits[:n_cand].cpu().numpy()
            l2, mx = check_close(got_logits, ref_logits, tol, f"step {t} logits", float_asserts)
            worst["logits"] = max(worst["logits"], l2, mx)
        ref_conf = np.concatenate(log.cand_conf)
        ref_tok = np.concatenate(log.cand_tok)
        l2, mx = check_close(cconf, ref_conf, 4 * tol, f"step {t} confidence", float_asserts)
        worst["conf"] = max(worst["conf"], l2, mx)
        # arg max: identical, or the oracle's own logits of the two tokens are within tolerance
        for i in np.nonzero(ctok != ref_tok)[0]:
            gap = abs(ref_logits[i, ctok[i]] - ref_logits[i, ref_tok[i]])
            if float_asserts:
                assert gap <= tol * np.max(np.abs(ref_logits[i])), f"step {t} cand {i}: token {ctok[i]} vs {ref_tok[i]}, gap {gap}"
            assert model.dtype == BF16, "fp32 mode must reproduce the oracle's tokens"
        if check_hidden:
            h = g.read_hidden()
            l2, mx = check_close(h, log.hidden, tol, f"step {t} hidden", float_asserts)
            worst["hidden"] = max(worst["hidden"], l2, mx)
        if per_block:
            p64, o64 = want_pos.astype(np.int64), want_off.astype(int)
            for l in range(model.n_layers):
                h_in = g.read_hidden(l).astype(np.float64)
                h_out = g.read_hidden(l + 1)
                Kl = g.k_cache[l].float().cpu().numpy().astype(np.float64)
                Vl = g.v_cache[l].float().cpu().numpy().astype(np.float64)
                K_dev, V_dev = Kl.copy(), Vl.copy()
                ref = OM.layer_forward(model, synth.layer(l), h_in, p64, o64, Kl, Vl)
                worst["block_out"] = max(worst["block_out"], *check_close(h_out, ref, tol, f"step {t} block {l} output rows"))
                for b in range(B):
                    pb = p64[o64[b]:o64[b + 1]]
                    if len(pb):
                        worst["block_kv"] = max(worst["block_kv"],
                                                *check_close(K_dev[b][:, pb], Kl[b][:, pb], tol, f"step {t} block {l} stored K rows"),
                                                *check_close(V_dev[b][:, pb], Vl[b][:, pb], tol, f"step {t} block {l} stored V rows"))
            # the head on the device's own final rows: the row of candidate q is q itself, or q - 1 under shifted logits
            rows_of = []
            for b in range(B):
                act = list(log.active[b])
                rows_of += [o64[b] + act.index(q - (1 if run.shift_logits else 0)) for q in log.cand[b]]
            head_ref = OM.logits_of(model, synth, h_out.astype(np.float64)[rows_of])
            if with_logits:
                worst["head_logits"] = max(worst["head_logits"], *check_close(got_logits, head_ref, tol, f"step {t} head logits"))
            htok, hconf = SA.predict(head_ref, model.mask_id)
            worst["head_conf"] = max(worst["head_conf"], *check_close(cconf, hconf, 4 * tol, f"step {t} head confidence"))
            for i in np.nonzero(ctok != htok)[0]:
                gap = abs(head_ref[i, ctok[i]] - head_ref[i, htok[i]])
                assert gap <= tol * np.max(np.abs(head_ref[i])), f"step {t} cand {i}: token {ctok[i]} vs {htok[i]}, gap {gap}"
        dpos = g.decoded_pos[t].cpu().numpy()
        dtok = g.decoded_tok[t].cpu().numpy()
        if teacher_forced or model.dtype == FP32:
            assert np.array_equal(dpos, log.pos), f"step {t}: committed positions {dpos} != {log.pos}"
            assert np.array_equal(dtok, log.tok), f"step {t}: committed tokens differ"
        else:
            raise AssertionError("free-running bf16 comparison is not meaningful")
        if verbose:
            print(f"step {t}: rows {len(want_pos)} cands {n_cand} worst {worst}", flush=True)
    assert np.array_equal(g.tokens.cpu().numpy(), st.tokens)
    assert np.array_equal(g.masked.cpu().numpy().astype(bool), st.masked)
    assert np.array_equal(g.stamp.cpu().numpy(), st.store.stamp)
    # cache contents: every row ever written, against the oracle's store
    Kg = g.k_cache.float().cpu().numpy()
    Vg = g.v_cache.float().cpu().numpy()
    worst["k_cache"] = max(check_close(Kg, st.store.K, tol, "K cache", float_asserts))
    worst["v_cache"] = max(check_close(Vg, st.store.V, tol, "V cache", float_asserts))
    return g, st, worst
