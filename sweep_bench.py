"""Throughput sweeps of the dKV-Cache path on synthetic shapes.

The paper's ablations vary the refresh interval (Sec. 4.3, "impact of the refresh interval"), the
one-step delay (Eq. 3 against Eq. 4), the prefill and decode lengths and the batch size (Appendix D), and
compare against decoding several tokens per step. This tool times whole generations of a depth-reduced,
full-width LLaDA-8B-shaped model (random weights: speed only, nothing is checked here) over those axes and
prints generated tokens/s, time per step and the cache ratio (share of the B x L rows per step that are
reused instead of recomputed, averaged over the steps).

    python sweep_bench.py --layers 4
"""
import argparse
import os
import sys
from dataclasses import replace

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))   # runnable from any cwd


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=4, help="transformer layers kept (full width)")
    ap.add_argument("--reps", type=int, default=2, help="timed generations per setting")
    ap.add_argument("--axes", default="interval,batch,k,decode_len,prefill_len,variant")
    args = ap.parse_args()
    import torch
    import dkv_inputs as D
    from dkv_inputs import configs as CF
    from paper_2505_15781_amd import binding

    model, base, wseed, pseed, _ = D.model_run(2)
    model = model.with_layers(args.layers)
    torch.cuda.set_device(0)
    weights = binding.random_weights(model, wseed)

    def measure(run, label):
        prompt = D.prompt_tokens(model, run, pseed)
        order = D.random_block_order(run, 77) if run.remask == CF.RANDOM_ORDER else None
        r = binding.DkvRun(model, run, weights, prompt, order=order)
        rows = 0
        for t in range(run.steps):                    # untimed pass: row counts of the schedule, warm-up
            rows += r.select_active(t)
            r.denoise_step(t)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ms = 0.0
        for _ in range(args.reps):
            r.reset()
            torch.cuda.synchronize()
            e0.record()
            r.generate()
            e1.record()
            torch.cuda.synchronize()
            ms += e0.elapsed_time(e1)
        ms /= args.reps
        ratio = 1.0 - rows / (run.steps * run.batch * run.seq_len)
        print(f"{label:44s} B={run.batch:3d} P={run.prompt_len:5d} G={run.gen_len:5d} T={run.steps:4d} "
              f"{run.batch * run.gen_len / ms * 1e3:9.1f} tok/s {ms / run.steps:8.3f} ms/step  cache ratio {ratio:5.3f}",
              flush=True)
        r.close()
        del r
        torch.cuda.empty_cache()

    axes = args.axes.split(",")
    print(f"# LLaDA-8B-shaped model cut to {args.layers} layers, bf16; tokens/s = B*G / generation time", flush=True)
    if "interval" in axes:
        for delay in (1, 0):
            for n in (1, 2, 4, 8, 16, 32, 1 << 30):
                name = "no cache (refresh every step)" if n == 1 else ("never refreshed" if n == 1 << 30 else f"refresh interval {n}")
                measure(replace(base, refresh_interval=n, delay=delay), f"decode, delay={delay}, {name}")
    if "batch" in axes:
        for b in (1, 2, 4, 8, 16, 32):
            measure(replace(base, batch=b), "decode, interval 8, batch size")
            measure(replace(base, batch=b, refresh_interval=1), "no cache, batch size")
    if "k" in axes:
        for k in (1, 2, 4):
            measure(replace(base, steps=base.gen_len // k), f"decode, interval 8, {k} tokens per step")
    if "decode_len" in axes:
        for g in (128, 256, 512, 1024):
            measure(replace(base, gen_len=g, steps=g), "decode, interval 8, decode length")
    if "prefill_len" in axes:
        for p in (128, 512, 1024, 2048):
            measure(replace(base, prompt_len=p), "decode, interval 8, prefill length")
            measure(replace(base, prompt_len=p, variant=CF.PD, refresh_interval=4), "prefill+decode (PD), interval 4")
    if "variant" in axes:
        measure(replace(base, variant=CF.PREFILL), "prefill only")
        measure(replace(base, variant=CF.PD, refresh_interval=4), "prefill+decode (PD), interval 4")
        measure(replace(base, variant=CF.GREEDY, remask=CF.RANDOM_ORDER, window=4, refresh_interval=4),
                "greedy, window 4, interval 4, random order")
        measure(replace(base, variant=CF.GREEDY, remask=CF.RANDOM_ORDER, window=2, refresh_interval=2),
                "greedy, window 2, interval 2, random order")


if __name__ == "__main__":
    sys.exit(main())
