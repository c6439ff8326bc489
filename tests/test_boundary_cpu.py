"""CPU-side checks of the boundary: the library loads, exports every declared symbol, and rejects bad
descriptors without touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2505_15781_amd", "libdkv.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2505_15781_amd.build import build
        build()
    return C.CDLL(LIB)


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "dkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dkv_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_entry_point_is_exported(lib):
    names = _declared_functions()
    assert {"dkv_init_cache", "dkv_select_active", "dkv_denoise_step", "dkv_refresh", "dkv_attn_update",
            "dkv_workspace_bytes", "dkv_destroy", "dkv_last_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in dkv.h but not exported"


def test_workspace_size_and_descriptor_validation_need_no_gpu():
    import dkv_inputs as D
    from paper_2505_15781_amd import binding as b
    for i in (0, 2, 3, 4):
        m, r, *_ = D.model_run(i)
        md, rd = b.model_desc(m), b.run_desc(r, C.c_void_p(16) if r.remask else None)
        assert b.lib.dkv_workspace_bytes(C.byref(md), C.byref(rd)) > 0
    m, r, *_ = D.model_run(0)
    bad = D.RunShape(batch=1, prompt_len=4, gen_len=8, steps=8, block_len=3, refresh_interval=2)
    assert b.lib.dkv_workspace_bytes(C.byref(b.model_desc(m)), C.byref(b.run_desc(bad))) == 0
    md = b.model_desc(m)
    md.head_dim = 48
    assert b.lib.dkv_workspace_bytes(C.byref(md), C.byref(b.run_desc(r))) == 0
    ctx = C.c_void_p()
    rc = b.lib.dkv_init_cache(C.byref(ctx), C.byref(md), None, None, None, None)
    assert rc == -1 and b.last_error()


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "one GPU" in res.stderr


def test_projection_and_attention_planners_return_sane_workspace_sizes_without_a_gpu():
    """The planners are host code: every (rows, shape) gets a K split from the documented set (the workspace is
    that many fp32 copies of the output), and the attention workspace never exceeds one partial record per
    (row, head, key slice) with at most seq_len / 64 slices."""
    from paper_2505_15781_amd import binding as b
    shapes = [(12288, 4096), (4096, 4096), (24576, 4096), (4096, 12288), (4608, 3584), (37888, 3584),
              (3584, 18944), (126464, 4096), (384, 128), (200, 136)]
    for n, k in shapes:
        for m in (1, 2, 17, 64, 65, 128, 129, 257, 512, 777, 1536, 4112, 12288):
            nb = b.lib.dkv_gemm_workspace_bytes(m, n, k, b.BF16)
            assert nb % (4 * m * n) == 0
            assert nb // (4 * m * n) in (0, 2, 3, 4, 6, 8), (m, n, k, nb)
            assert b.lib.dkv_gemm_workspace_bytes(m, n, k, b.FP32) == 0
    assert b.lib.dkv_gemm_workspace_bytes(0, 128, 64, b.BF16) == 0
    for (B, hq, hkv, L, dh) in [(8, 32, 32, 1024, 128), (1, 32, 32, 512, 128), (4, 32, 32, 1536, 128),
                                (16, 28, 4, 768, 128), (3, 6, 2, 203, 64), (1, 4, 2, 2085, 128)]:
        for rows in (1, 5, 16, 64, 257, L):
            nb = b.lib.dkv_attn_update_workspace_bytes(B, hq, hkv, L, dh, b.BF16, rows)
            g = hq // hkv
            rows_pad = -(-(-(-rows * g // 16) * 16) // g)
            assert nb <= B * rows_pad * hq * max(1, L // 64) * (dh + 4) * 4, (B, hq, hkv, L, dh, rows, nb)
        assert b.lib.dkv_attn_update_workspace_bytes(B, hq, hkv, L, dh, b.FP32, 8) <= 256     # no partial records


def test_kernel_kind_numbers_of_the_header_and_the_binding_agree():
    """The profile report is indexed by the kind numbers of dkv.h; the binding names them in the same order."""
    text = open(os.path.join(ROOT, "include", "dkv.h")).read()
    defs = {m.group(1): int(m.group(2)) for m in re.finditer(r"#define\s+(DKV_(?:GEMM|PROF)_[A-Za-z0-9_]+)\s+(\d+)\b", text)}
    src = open(os.path.join(ROOT, "paper_2505_15781_amd", "binding.py")).read()
    kinds = eval(re.search(r"^GEMM_KINDS = (\{.*?\})", src, flags=re.S | re.M).group(1))
    names = eval(re.search(r"^PROF_KINDS = (\(.*?\))\n", src, flags=re.S | re.M).group(1))
    assert len(names) == defs["DKV_PROF_KINDS"] and names[defs["DKV_PROF_ATTN"]] == "attention"
    for name, number in kinds.items():
        tag = name.upper().replace("X", "x")
        assert defs["DKV_GEMM_" + tag] == number, name
    # every projection kind of the header has a name in the binding, and the tile kinds carry their template arguments
    assert sorted(kinds.values()) == list(range(defs["DKV_PROF_ATTN"]))
    tiles = {m.group(1): (int(m.group(2)), int(m.group(3))) for m in re.finditer(r"(DKV_GEMM_DMA_(\d+)x(\d+))", text)}
    for tag, (rows, cols) in tiles.items():
        mt, nt, wm, wn = (int(x) for x in re.match(r"gemm_dma<\*,(\d),(\d),(\d),(\d),\d>", names[defs[tag]]).groups())
        assert (32 * mt * wm, 32 * nt * wn) == (rows, cols), tag
