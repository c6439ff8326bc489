"""Microbenchmark of the projection kernel on the layer shapes of a model configuration.

Runs y = x W^T through the library (`dkv_gemm`, heuristic kernel choice) for the four projections of
one transformer layer at a sample of the row counts a dKV-Cache-Decode schedule produces, rotating
over enough weight buffers that every launch streams its weights from HBM. Used on its own for
kernel timing and under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` for HBM traffic per launch
(`--copy-calibration` adds one elementwise kernel that reads and writes exactly 1 GiB).

    python kernel_bench.py --config 2 --rows 2,32,64,128,192,256,512
"""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))   # runnable from any cwd


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 4])
    ap.add_argument("--rows", default="2,32,64,128,192,256,512")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--copy-calibration", action="store_true")
    ap.add_argument("--attention", default=None, metavar="ROWS",
                    help="instead: time cache update + attention at the configs[1] shape for these active rows per "
                         "sequence (e.g. 1,8,32,128,512), over rotating caches larger than the last-level cache")
    ap.add_argument("--peaks", action="store_true",
                    help="instead: what the chip sustains on the yardstick kernels (cold streaming read, plain copy, "
                         "register-only bf16 MFMA loop)")
    ap.add_argument("--layout-alternative", action="store_true",
                    help="instead: time the compact-layout concat_reorder operator of the paper's Appendix A per layer-step")
    args = ap.parse_args()
    import torch
    import dkv_inputs as D
    from paper_2505_15781_amd import binding
    from paper_2505_15781_amd.binding import lib, _ptr, _stream, _check

    torch.cuda.set_device(0)
    if args.copy_calibration:         # peak_copy_kernel: reads exactly 1 GiB and writes exactly 1 GiB
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        _check(lib.dkv_peak_copy(_ptr(src), _ptr(dst), 1 << 30, _stream()))
        torch.cuda.synchronize()
        del src, dst
    if args.peaks:
        print(binding.measured_peaks(), flush=True)
        return 0
    if args.layout_alternative:
        return layout_alternative(torch, binding)
    if args.attention:
        return attention(torch, D, [int(a) for a in args.attention.split(",")], args.reps)
    model = D.model_run(args.config)[0]
    d, F = model.d_model, model.d_ffn
    shapes = {"qkv": (model.qkv_rows, d), "o": (d, model.n_q_heads * model.head_dim), "gate_up": (2 * F, d),
              "down": (d, F)}
    torch.cuda.set_device(0)
    g = torch.Generator(device="cuda").manual_seed(1)
    for name, (N, K) in shapes.items():
        nbuf = max(2, int(600e6 // (N * K * 2)) + 1)
        Ws = [(torch.randn(N, K, generator=g, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(nbuf)]
        for M in [int(r) for r in args.rows.split(",")]:
            x = torch.randn(M, K, generator=g, device="cuda").to(torch.bfloat16)
            y = torch.empty(M, N, device="cuda", dtype=torch.float32)
            nb = lib.dkv_gemm_workspace_bytes(M, N, K, binding.BF16)
            ws = torch.empty(max(nb, 4), dtype=torch.uint8, device="cuda")

            def run(w):
                _check(lib.dkv_gemm(_ptr(x), _ptr(w), _ptr(y), M, N, K, binding.BF16, _ptr(ws), nb, _stream()))

            for _ in range(3):                 # warm-up: clocks and caches in the state of a running model
                for w in Ws:
                    run(w)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.reps):
                for w in Ws:
                    run(w)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / (args.reps * nbuf)
            nbytes = (M * K + N * K) * 2 + 4 * M * N
            print(f"{name:8s} M={M:5d} N={N:6d} K={K:6d} k_slices={max(1, nb // (4 * M * N))} {us:8.1f} us "
                  f"{nbytes / us * 1e-3:7.0f} GB/s {2.0 * M * N * K / us * 1e-6:7.1f} TFLOP/s", flush=True)
        del Ws
        torch.cuda.empty_cache()


def attention(torch, D, sizes, reps):
    """dkv_attn_update at B=8, 32 heads x 128, L=1024: per call the 134 MB of K/V are read once from HBM."""
    import paper_2505_15781_amd as P
    torch.cuda.set_device(0)
    shape = D.CONFIG1_SHAPE
    B, H, L, dh = shape.batch, shape.n_q_heads, shape.seq_len, shape.head_dim
    nbuf = 5
    g = torch.Generator(device="cuda").manual_seed(1100)
    kc = [torch.randn((B, H, L, dh), generator=g, device="cuda").to(torch.bfloat16) for _ in range(nbuf)]
    vc = [torch.randn((B, H, L, dh), generator=g, device="cuda").to(torch.bfloat16) for _ in range(nbuf)]
    for i, A in enumerate(sizes):
        c = D.attn_update_case(D.AttnUpdateShape(B, 1, 1, L, 2), A, 1100 + i)     # positions only
        idx, off = torch.from_numpy(c["active_idx"]).cuda(), torch.from_numpy(c["active_off"]).cuda()
        R = B * A
        q, kn, vn = (torch.randn((R, H, dh), generator=g, device="cuda").to(torch.bfloat16) for _ in range(3))
        o = torch.empty_like(q)
        ws = torch.empty(max(P.attn_update_workspace_bytes(B, H, H, L, dh, P.BF16, A), 256), dtype=torch.uint8,
                         device="cuda")
        for j in range(nbuf):
            P.attn_update(kc[j], vc[j], q, kn, vn, idx, off, o, R, A, P.BF16, ws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            for j in range(nbuf):
                P.attn_update(kc[j], vc[j], q, kn, vn, idx, off, o, R, A, P.BF16, ws)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (reps * nbuf)
        nbytes = 2 * B * H * L * dh * 2 + 6 * R * H * dh * 2
        print(f"active rows {A:4d}: {us:8.1f} us {nbytes / us * 1e-3:7.0f} GB/s "
              f"{4.0 * R * H * L * dh / us * 1e-6:7.1f} TFLOP/s", flush=True)


def layout_alternative(torch, binding):
    """One layer-step of concat_reorder at the four workloads' cache shapes (cached rows of every sequence and
    head are copied into the next order), over rotating buffers larger than the last-level cache."""
    torch.cuda.set_device(0)
    shapes = {"configs[1] A=8": (8, 32, 1024, 8), "configs[2] step 128": (1, 32, 512, 129),
              "configs[3] greedy step": (4, 32, 1536, 7), "configs[4] step 128": (16, 4, 768, 129)}
    g = torch.Generator(device="cuda").manual_seed(2)
    for name, (B, H, L, n_new) in shapes.items():
        n_c = L - n_new
        per = 2 * B * H * L * 128 * 2
        nbuf = max(2, int(600e6 // per) + 1)
        bufs = [tuple(torch.randn((B, H, n, 128), generator=g, device="cuda").to(torch.bfloat16)
                      for n in (n_c, n_c, n_new, n_new)) for _ in range(nbuf)]
        take = torch.stack([torch.randperm(L, generator=g, device="cuda") for _ in range(B)]).to(torch.int32)
        for kc, vc, kn, vn in bufs:
            binding.concat_reorder(kc, vc, kn, vn, take, binding.BF16)
        torch.cuda.synchronize()
        k_out = torch.empty((B, H, L, 128), dtype=torch.bfloat16, device="cuda")
        v_out = torch.empty_like(k_out)
        from paper_2505_15781_amd.binding import lib, _ptr, _stream, _check
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        reps = 10
        for _ in range(reps):
            for kc, vc, kn, vn in bufs:
                _check(lib.dkv_concat_reorder(_ptr(kc), _ptr(vc), _ptr(kn), _ptr(vn), _ptr(take), _ptr(k_out),
                                              _ptr(v_out), B, H, n_c, n_new, 128, binding.BF16, _stream()))
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (reps * nbuf)
        print(f"{name:24s} B={B:2d} Hkv={H:2d} L={L:5d} new rows {n_new:4d}: {us:7.1f} us per layer-step, "
              f"{2 * per / us * 1e-3:6.0f} GB/s read+write; the position-indexed cache writes "
              f"{2 * B * H * n_new * 256 / 1e3:.0f} KB in the RoPE kernel instead", flush=True)


if __name__ == "__main__":
    sys.exit(main())
