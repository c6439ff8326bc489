"""GPU parity of the isolated kernels (projection, cache update + attention) against the oracle."""
import numpy as np
import pytest
import torch

import dkv_inputs as D
from dkv_inputs.configs import BF16, FP32
from oracle.attn_update import attn_update as oracle_attn_update
from helpers import rel_err
from gpu_parity import check_close, tolerances

pytestmark = pytest.mark.gpu


def _dev(x, dtype):
    td = torch.bfloat16 if dtype == BF16 else torch.float32
    return torch.from_numpy(np.ascontiguousarray(x)).to(device="cuda", dtype=td)


@pytest.mark.parametrize("dtype", [BF16, FP32])
@pytest.mark.parametrize("m,n,k", [(1, 128, 64), (2, 384, 4096), (37, 200, 136), (64, 256, 512),
                                   (129, 384, 1024), (300, 130, 72), (513, 256, 256)])
def test_projection_matches_float64_product(dtype, m, n, k):
    import paper_2505_15781_amd as P
    x = D.normal_f32(5, 1, (m, k), bf16=dtype == BF16)
    w = D.normal_f32(5, 2, (n, k), std=0.02, bf16=dtype == BF16)
    y = P.gemm(_dev(x, dtype), _dev(w, dtype), dtype).cpu().numpy()
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    check_close(y, ref, 1e-5, f"gemm {m}x{n}x{k}")


@pytest.mark.parametrize("m", [3, 40, 100])
def test_projection_planned_launch_on_a_weight_matrix_that_is_streamed(m):
    """A weight matrix of 32 MB: with one row of tiles the planner streams it with the non-temporal hint, slices K
    and staggers the K start; the product is the same."""
    import paper_2505_15781_amd as P
    n, k = 4096, 4096
    x = D.normal_f32(7, 1, (m, k), bf16=True)
    w = D.normal_f32(7, 2, (n, k), std=0.02, bf16=True)
    y = P.gemm(_dev(x, BF16), _dev(w, BF16), BF16).cpu().numpy()
    check_close(y, x.astype(np.float64) @ w.astype(np.float64).T, 1e-5, f"gemm {m}x{n}x{k}")


@pytest.mark.parametrize("kind,split", [("dma_32x128", 1), ("dma_32x128", 3), ("dma_64x128", 2), ("dma_128x128", 1),
                                        ("dma_128x128", 4), ("dma_128x256", 2), ("dma_256x256", 1),
                                        ("dma_256x256", 3), ("dma_128x96", 1), ("dma_128x96", 2),
                                        ("dma_128x192", 1), ("dma_128x192", 3), ("dma_256x192", 1), ("dma_256x192", 2),
                                        ("dma_192x256", 1), ("dma_192x256", 2),
                                        ("reg_64x128", 2)])
@pytest.mark.parametrize("m,n,k", [(1, 128, 64), (37, 200, 192), (129, 384, 1024), (300, 520, 640), (513, 256, 2048)])
def test_every_projection_kernel_on_ragged_shapes(kind, split, m, n, k):
    import paper_2505_15781_amd as P
    if split > max(1, k // 64):
        pytest.skip("more K slices than K tiles")
    x = D.normal_f32(6, 1, (m, k), bf16=True)
    w = D.normal_f32(6, 2, (n, k), std=0.02, bf16=True)
    # the effective number of slices may be smaller than requested; ask the library's own count
    kt = -(-k // 64)
    kps = -(-kt // split)
    split_eff = -(-kt // kps)
    y = P.gemm(_dev(x, BF16), _dev(w, BF16), BF16, kind=kind, split_k=split_eff).cpu().numpy()
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    check_close(y, ref, 1e-5, f"{kind} split {split_eff} {m}x{n}x{k}")


@pytest.mark.parametrize("kind", ["dma_32x128", "dma_64x128", "dma_128x128", "dma_128x256", "dma_256x256",
                                  "dma_128x96", "dma_128x192", "dma_256x192", "dma_192x256"])
@pytest.mark.parametrize("options", [1, 2, 3, 8, 9])
@pytest.mark.parametrize("m,n,k,split", [(5, 128, 256, 1), (129, 384, 1024, 1), (300, 520, 768, 2),
                                         (1100, 1536, 512, 1), (1030, 2048, 640, 2)])
def test_projection_launch_options_leave_the_product_unchanged(kind, options, m, n, k, split):
    """A staggered K loop start and the XCD-grouped tile order only permute work: same product (up to fp32
    summation order); the last two shapes have at least four tile rows, so the grouping is really applied."""
    import paper_2505_15781_amd as P
    x = D.normal_f32(9, 1, (m, k), bf16=True)
    w = D.normal_f32(9, 2, (n, k), std=0.02, bf16=True)
    y = P.gemm(_dev(x, BF16), _dev(w, BF16), BF16, kind=kind, split_k=split, options=options).cpu().numpy()
    check_close(y, x.astype(np.float64) @ w.astype(np.float64).T, 1e-5, f"{kind} options {options} {m}x{n}x{k}")


@pytest.mark.parametrize("kind", ["dma_32x128", "dma_64x128", "dma_128x128", "dma_128x256", "dma_256x256",
                                  "dma_128x96", "dma_128x192", "dma_256x192", "dma_192x256"])
@pytest.mark.parametrize("m,n,k", [(5, 128, 256), (129, 392, 1024), (300, 520, 768)])
def test_projection_with_fused_swiglu_epilogue(kind, m, n, k):
    """Rows of w interleave gate_j, up_j; the epilogue writes silu(gate) * up (the feed-forward's activation)
    as bf16 [m, n/2] instead of the fp32 product. bf16 output: one rounding, 2^-9 relative."""
    import paper_2505_15781_amd as P
    from paper_2505_15781_amd import binding
    x = D.normal_f32(10, 1, (m, k), bf16=True)
    w = D.normal_f32(10, 2, (n, k), std=0.05, bf16=True)
    y = P.gemm(_dev(x, BF16), _dev(w, BF16), BF16, kind=kind, split_k=1,
               options=binding.GEMM_OPT_SWIGLU).float().cpu().numpy()
    prod = x.astype(np.float64) @ w.astype(np.float64).T
    g, u = prod[:, 0::2], prod[:, 1::2]
    check_close(y, g / (1.0 + np.exp(-g)) * u, 4e-3, f"{kind} fused swiglu {m}x{n}x{k}")
    with pytest.raises(P.DkvError) as e:
        P.gemm(_dev(x, BF16), _dev(w, BF16), BF16, kind=kind, split_k=2, options=binding.GEMM_OPT_SWIGLU)
    assert e.value.code == -3


def test_projection_rejects_unknown_option_bits():
    import paper_2505_15781_amd as P
    x = _dev(D.normal_f32(6, 1, (4, 64), bf16=True), BF16)
    w = _dev(D.normal_f32(6, 2, (8, 64), bf16=True), BF16)
    with pytest.raises(P.DkvError) as e:
        P.gemm(x, w, BF16, kind="dma_32x128", split_k=1, options=16)
    assert e.value.code == -1


@pytest.mark.parametrize("kind", ["dma_32x128", "dma_64x128", "dma_128x128", "dma_128x256", "dma_256x256"])
@pytest.mark.parametrize("m,n,k", [(5, 128, 256), (37, 200, 512), (129, 384, 1024), (300, 520, 768), (257, 1536, 4096)])
def test_three_quarter_k_share_covers_every_tile_twice(kind, m, n, k):
    """Workgroups that take 3/4 of a tile's K range each (possibly ending one tile and starting the next)."""
    import paper_2505_15781_amd as P
    x = D.normal_f32(8, 1, (m, k), bf16=True)
    w = D.normal_f32(8, 2, (n, k), std=0.02, bf16=True)
    y = P.gemm(_dev(x, BF16), _dev(w, BF16), BF16, kind=kind, split_k=-1).cpu().numpy()
    check_close(y, x.astype(np.float64) @ w.astype(np.float64).T, 1e-5, f"{kind} 3/4 share {m}x{n}x{k}")


def test_projection_kernel_rejects_shapes_it_cannot_take():
    import paper_2505_15781_amd as P
    x = _dev(D.normal_f32(6, 1, (4, 72), bf16=True), BF16)
    w = _dev(D.normal_f32(6, 2, (8, 72), bf16=True), BF16)
    with pytest.raises(P.DkvError) as e:
        P.gemm(x, w, BF16, kind="dma_128x128", split_k=1)      # K = 72 is not a multiple of 64
    assert e.value.code == -3
    y = P.gemm(x, w, BF16, kind="reg_64x128", split_k=1).cpu().numpy()
    check_close(y, x.float().cpu().numpy().astype(np.float64) @ w.float().cpu().numpy().astype(np.float64).T, 1e-5, "reg")


def _attn_case(shape, n_active, seed, ragged=None, q_scale=1.0):
    import paper_2505_15781_amd as P
    c = D.attn_update_case(shape, n_active, seed, ragged=ragged)
    c["q"] = c["q"] * np.float32(q_scale)            # a power of two: still exact bfloat16 values
    dt = shape.dtype
    kc, vc = _dev(c["k_cache"], dt), _dev(c["v_cache"], dt)
    rows = int(c["active_off"][-1])
    max_rows = int(np.max(np.diff(c["active_off"]))) if shape.batch else 0
    q, kn, vn = _dev(c["q"], dt), _dev(c["k_new"], dt), _dev(c["v_new"], dt)
    idx = torch.from_numpy(c["active_idx"]).cuda()
    off = torch.from_numpy(c["active_off"]).cuda()
    out = torch.zeros((max(rows, 1), shape.n_q_heads, shape.head_dim), dtype=q.dtype, device="cuda")
    nb = P.attn_update_workspace_bytes(shape.batch, shape.n_q_heads, shape.n_kv_heads, shape.seq_len,
                                       shape.head_dim, dt, max_rows)
    ws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
    P.attn_update(kc, vc, q, kn, vn, idx, off, out, rows, max_rows, dt, ws)
    torch.cuda.synchronize()
    rk, rv = c["k_cache"].astype(np.float64), c["v_cache"].astype(np.float64)
    ref = oracle_attn_update(rk, rv, c["q"], c["k_new"], c["v_new"], c["active_idx"], c["active_off"])
    # the scatter is a copy: cache contents must be bit-exact
    assert np.array_equal(kc.float().cpu().numpy().astype(np.float64), rk)
    assert np.array_equal(vc.float().cpu().numpy().astype(np.float64), rv)
    if rows:
        check_close(out[:rows].float().cpu().numpy(), ref, tolerances(dt), f"attention A={n_active} {ragged}")


@pytest.mark.parametrize("dh", [128, 64])
def test_attention_small_ragged_gqa_bf16(dh):
    shape = D.AttnUpdateShape(batch=3, n_q_heads=6, n_kv_heads=2, seq_len=203, head_dim=dh, dtype=BF16)
    _attn_case(shape, None, 31, ragged=[5, 0, 37])
    _attn_case(shape, None, 32, ragged=[1, 1, 1])
    _attn_case(shape, None, 33, ragged=[203, 64, 17])


@pytest.mark.parametrize("dh", [128, 64])
def test_attention_key_slices_across_workgroups(dh):
    """Few (sequence, head) pairs and many keys: the keys are sliced over several workgroups and merged by
    the second kernel; 2085 keys leave a ragged last tile and an uneven deal of tiles to the wavefronts."""
    shape = D.AttnUpdateShape(batch=1, n_q_heads=4, n_kv_heads=2, seq_len=2085, head_dim=dh, dtype=BF16)
    _attn_case(shape, None, 34, ragged=[21])
    shape = D.AttnUpdateShape(batch=2, n_q_heads=2, n_kv_heads=2, seq_len=1031, head_dim=dh, dtype=BF16)
    _attn_case(shape, None, 35, ragged=[3, 40])


def test_attention_many_query_tiles_per_head():
    """Enough query rows per kv head for the kernel whose wavefronts share K/V tiles (GQA group of 8 and
    79 rows: 40 tiles = 5 full blocks of 8), and a count that leaves its last block almost empty (66 rows:
    33 tiles)."""
    shape = D.AttnUpdateShape(batch=16, n_q_heads=128, n_kv_heads=16, seq_len=300, head_dim=128, dtype=BF16)
    _attn_case(shape, 79, 36)
    _attn_case(shape, 66, 37)


@pytest.mark.parametrize("seq_len", [64, 100, 192, 300, 512])
def test_attention_shared_tiles_eight_wavefronts(seq_len):
    """Fewer than two workgroups per compute unit for the shared-tile kernel (4 x 16 kv heads x 5 blocks = 320):
    its 8-wavefront form, which keeps two tiles on their way. Key counts of 1, 2 (ragged), 3, 5 (ragged) and 8
    tiles take both exits of its two-tile loop; 66 rows leave the last block almost empty."""
    shape = D.AttnUpdateShape(batch=4, n_q_heads=128, n_kv_heads=16, seq_len=seq_len, head_dim=128, dtype=BF16)
    n = min(79, seq_len)
    _attn_case(shape, n, 44)
    _attn_case(shape, min(66, seq_len), 45)


def test_attention_shared_tiles_with_ragged_sequences():
    """Shared-tile kernel over sequences with no active row at all, with every position active (first and last
    included) and with a few: in its 8-wavefront form (one block of query tiles per (sequence, kv head), K/V
    fetched with the streaming hint) and in its 4-wavefront form (several blocks per pair)."""
    shape = D.AttnUpdateShape(batch=4, n_q_heads=64, n_kv_heads=64, seq_len=300, head_dim=128, dtype=BF16)
    _attn_case(shape, None, 52, ragged=[100, 0, 128, 5])
    shape = D.AttnUpdateShape(batch=4, n_q_heads=128, n_kv_heads=16, seq_len=300, head_dim=128, dtype=BF16)
    _attn_case(shape, None, 53, ragged=[79, 0, 300, 5])


@pytest.mark.parametrize("dh", [128, 64])
def test_attention_many_small_items(dh):
    """More (sequence, head, query group) items than compute units: the key-split kernel in its
    4-wavefront form, two workgroups per compute unit, with the cache update fused (40 rows per sequence)."""
    shape = D.AttnUpdateShape(batch=20, n_q_heads=16, n_kv_heads=16, seq_len=150, head_dim=dh, dtype=BF16)
    _attn_case(shape, 40, 38)


@pytest.mark.parametrize("q_scale", [16.0, 0.0])
def test_attention_peaked_and_flat_softmax(q_scale):
    """Scores with a standard deviation of 16 (after the 1/sqrt(d_h)): almost one-hot probabilities, running maxima
    that keep rising over the key tiles and rescale the output; and all-zero queries: every key weighs the same, the
    output is the mean of V. Through the key-split, both shared-tile and the generic kernels."""
    _attn_case(D.AttnUpdateShape(batch=2, n_q_heads=4, n_kv_heads=2, seq_len=1031, head_dim=128, dtype=BF16),
               None, 46, ragged=[3, 40], q_scale=q_scale)
    _attn_case(D.AttnUpdateShape(batch=4, n_q_heads=128, n_kv_heads=16, seq_len=300, head_dim=128, dtype=BF16),
               79, 47, q_scale=q_scale)
    _attn_case(D.AttnUpdateShape(batch=16, n_q_heads=128, n_kv_heads=16, seq_len=200, head_dim=128, dtype=BF16),
               66, 48, q_scale=q_scale)
    _attn_case(D.AttnUpdateShape(batch=2, n_q_heads=4, n_kv_heads=4, seq_len=70, head_dim=32, dtype=FP32),
               None, 49, ragged=[9, 33], q_scale=q_scale)


def test_attention_generic_paths():
    _attn_case(D.AttnUpdateShape(batch=2, n_q_heads=4, n_kv_heads=4, seq_len=70, head_dim=32, dtype=FP32),
               None, 41, ragged=[9, 33])
    _attn_case(D.AttnUpdateShape(batch=2, n_q_heads=4, n_kv_heads=2, seq_len=70, head_dim=32, dtype=BF16),
               None, 42, ragged=[9, 33])
    _attn_case(D.AttnUpdateShape(batch=1, n_q_heads=2, n_kv_heads=1, seq_len=40, head_dim=128, dtype=FP32),
               None, 43, ragged=[7])


def test_attention_no_rows_is_a_no_op():
    shape = D.AttnUpdateShape(batch=2, n_q_heads=4, n_kv_heads=2, seq_len=64, head_dim=128, dtype=BF16)
    _attn_case(shape, 0, 51)


@pytest.mark.parametrize("n_active", D.CONFIG1_ACTIVE_SIZES)
def test_attention_microbenchmark_configuration_full_size(n_active):
    _attn_case(D.CONFIG1_SHAPE, n_active, 1100 + D.CONFIG1_ACTIVE_SIZES.index(n_active))


@pytest.mark.parametrize("dtype", [BF16, FP32])
def test_concat_reorder_operator_reproduces_the_compact_layout(dtype):
    """The paper's cache operator (Appendix A) on its compact layout, bit for bit: cached rows left, new rows
    right, gathered into the next step's order given by the oracle's index bookkeeping (which the worked
    example of the appendix pins)."""
    import paper_2505_15781_amd as P
    from oracle import schedule as S
    B, H, L, dh = 3, 2, 23, 64
    rng = np.random.default_rng(5)
    full_k = D.normal_f32(12, 1, (B, H, L, dh), bf16=dtype == BF16)      # K/V of every position, position order
    full_v = D.normal_f32(12, 2, (B, H, L, dh), bf16=dtype == BF16)
    n_c = 9
    kc, vc, kn, vn, take, want_k, want_v = [], [], [], [], [], [], []
    for b in range(B):
        unm_prev = sorted(rng.choice(L, size=n_c, replace=False).tolist())            # cached at this step
        rest = [p for p in range(L) if p not in unm_prev]
        unm_next = sorted(unm_prev + rng.choice(rest, size=2, replace=False).tolist())   # two more next step
        layout_prev, layout_next, mapping, _ = S.reorder_map(unm_prev, unm_next, L)
        kc.append(full_k[b][:, layout_prev[:n_c]]); vc.append(full_v[b][:, layout_prev[:n_c]])
        kn.append(full_k[b][:, layout_prev[n_c:]]); vn.append(full_v[b][:, layout_prev[n_c:]])
        take.append(mapping)
        want_k.append(full_k[b][:, layout_next]); want_v.append(full_v[b][:, layout_next])
    dev = lambda xs: _dev(np.stack(xs), dtype)
    tk = torch.tensor(np.asarray(take, dtype=np.int32), device="cuda")
    ko, vo = P.concat_reorder(dev(kc), dev(vc), dev(kn), dev(vn), tk, dtype)
    assert np.array_equal(ko.float().cpu().numpy(), np.stack(want_k))
    assert np.array_equal(vo.float().cpu().numpy(), np.stack(want_v))


def test_bad_arguments_are_errors_not_faults():
    import paper_2505_15781_amd as P
    shape = D.AttnUpdateShape(batch=1, n_q_heads=2, n_kv_heads=1, seq_len=40, head_dim=48, dtype=BF16)
    kc = torch.zeros((1, 1, 40, 48), dtype=torch.bfloat16, device="cuda")
    q = torch.zeros((1, 2, 48), dtype=torch.bfloat16, device="cuda")
    kn = torch.zeros((1, 1, 48), dtype=torch.bfloat16, device="cuda")
    idx = torch.zeros(1, dtype=torch.int32, device="cuda")
    off = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    with pytest.raises(P.DkvError) as e:
        P.attn_update(kc, kc.clone(), q, kn, kn, idx, off, q.clone(), 1, 1, BF16, None)
    assert e.value.code == -3 and "head_dim" in str(e.value)


def test_yardstick_kernels_copy_exactly_and_report_their_flops():
    """The benchmark's yardsticks: the copy kernel moves every byte (it calibrates the HBM byte counters), the MFMA loop
    reports the flops of its launch, and the three measured rates are of the chip's order of magnitude."""
    import ctypes as C
    from paper_2505_15781_amd import binding as b
    n = (1 << 20) + 48
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    b._check(b.lib.dkv_peak_copy(b._ptr(src), b._ptr(dst), n, b._stream()))
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert b.lib.dkv_peak_copy(b._ptr(src), b._ptr(dst), n - 1, b._stream()) == -1      # not a multiple of 16 bytes
    sink = torch.zeros(1 << 21, dtype=torch.uint8, device="cuda")
    flops = C.c_double(0.0)
    b._check(b.lib.dkv_peak_mfma(b._ptr(sink), 10, C.byref(flops), b._stream()))
    torch.cuda.synchronize()
    assert flops.value == 2048 * 4 * 10 * 4 * 2.0 * 32 * 32 * 16 and not sink.any()
    p = b.measured_peaks(reps=2)
    assert 1000 < p["hbm_read_GBps"] < 8000 and 1000 < p["hbm_copy_GBps"] < 8000 and 300 < p["mfma_bf16_TFLOPs"] < 2600


def test_profile_report_counts_the_bytes_each_projection_really_moves():
    """dkv_profile_begin / end: per kernel kind launches and algorithmic bytes and flops; gate/up with the fused
    SwiGLU counts its bf16 [M, N/2] output, the vocabulary projection none (its epilogue keeps statistics only)."""
    import paper_2505_15781_amd as P
    from paper_2505_15781_amd import binding
    from dkv_inputs.configs import ModelShape, RunShape
    m = ModelShape(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=384, vocab=520, mask_id=519,
                   dtype=BF16)
    r = RunShape(batch=2, prompt_len=8, gen_len=8, steps=8, block_len=8, refresh_interval=4)
    g = P.DkvRun(m, r, binding.random_weights(m, 3), D.prompt_tokens(m, r, 4))
    g.profile_begin()
    g.denoise_step(0)
    prof = g.profile_end()
    rows, cands, d, F, V = 2 * 16, 2 * 8, m.d_model, m.d_ffn, m.vocab
    nqkv, qn = m.qkv_rows, m.n_q_heads * m.head_dim
    proj = lambda M, N, K, out: (M * K + N * K) * 2 + out
    want_bytes = m.n_layers * (proj(rows, nqkv, d, 4 * rows * nqkv) + proj(rows, d, qn, 4 * rows * d) +
                               proj(rows, 2 * F, d, 2 * rows * F) + proj(rows, d, F, 4 * rows * d)) + proj(cands, V, d, 0)
    want_flops = m.n_layers * 2.0 * rows * d * (nqkv + qn + 2 * F + F) + 2.0 * cands * V * d
    got = [v for k, v in prof.items() if k != "attention" and v["launches"]]
    assert sum(v["launches"] for v in got) == 4 * m.n_layers + 1
    assert sum(v["bytes"] for v in got) == want_bytes and sum(v["flops"] for v in got) == want_flops
    assert prof["attention"]["launches"] == m.n_layers
    g.close()
