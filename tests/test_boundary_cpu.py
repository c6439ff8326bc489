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
