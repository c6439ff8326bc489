"""MI355X-native dKV-Cache hot path (arxiv 2505.15781): HIP library + thin ctypes binding.

The binding (and with it libdkv.so) is loaded on first use of one of the names below, so that
`python -m paper_2505_15781_amd.build` can (re)build the library when none, or a stale one, is there.
"""
_BINDING_NAMES = ("lib", "DkvError", "DkvRun", "attn_update", "attn_update_static", "attn_update_workspace_bytes",
                  "gemm", "GEMM_KINDS", "concat_reorder", "BF16", "FP32", "last_error")


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding":
        import importlib
        binding = importlib.import_module(".binding", __name__)
        return binding if name == "binding" else getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
