"""ctypes binding of libdkv.so: argument marshalling only, every step runs in the HIP kernels.

PyTorch supplies device memory and the stream. The library must have been built
(`python -m paper_2505_15781_amd.build`); importing this module without it raises.
"""
import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdkv.so")
BF16, FP32 = 0, 1

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_15781_amd.build` "
                      "(there is no CPU fallback)")
lib = C.CDLL(LIB_PATH)

c_i32, c_f32, c_vp, c_sz = C.c_int32, C.c_float, C.c_void_p, C.c_size_t


class ModelDesc(C.Structure):
    _fields_ = [(n, c_i32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn",
                                     "vocab", "mask_id", "dtype")] + [("rms_eps", c_f32), ("rope_theta", c_f32)]


class Weights(C.Structure):
    _fields_ = [("embed", c_vp), ("lm_head", c_vp), ("final_norm", c_vp)] + \
               [(n, C.POINTER(c_vp)) for n in ("wqkv", "wo", "w_gate_up", "w_down", "norm1", "norm2")]


class RunDesc(C.Structure):
    _fields_ = [(n, c_i32) for n in ("batch", "prompt_len", "gen_len", "steps", "block_len", "refresh_interval",
                                     "variant", "delay", "window", "window_center", "include_prev", "remask",
                                     "shift_logits")] + \
               [("order", c_vp)]


class Buffers(C.Structure):
    _fields_ = [(n, c_vp) for n in ("k_cache", "v_cache", "tokens", "masked", "stamp", "decoded_pos",
                                    "decoded_tok", "decoded_conf", "workspace")] + [("workspace_bytes", c_sz)]


lib.dkv_last_error.restype = C.c_char_p
lib.dkv_workspace_bytes.restype = c_sz
lib.dkv_workspace_bytes.argtypes = [C.POINTER(ModelDesc), C.POINTER(RunDesc)]
lib.dkv_init_cache.argtypes = [C.POINTER(c_vp), C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(RunDesc),
                               C.POINTER(Buffers), c_vp]
lib.dkv_select_active.argtypes = [c_vp, c_i32, c_vp, c_vp, C.POINTER(c_i32)]
lib.dkv_denoise_step.argtypes = [c_vp, c_i32, c_vp, c_vp, c_vp]
lib.dkv_refresh.argtypes = [c_vp, c_i32]
lib.dkv_read_rows.argtypes = [c_vp, c_vp, c_vp, c_i32, C.POINTER(c_i32)]
lib.dkv_read_candidates.argtypes = [c_vp, c_vp, c_vp, c_vp, c_vp, c_i32, C.POINTER(c_i32)]
lib.dkv_read_hidden.argtypes = [c_vp, c_i32, c_vp, c_i32, C.POINTER(c_i32)]
lib.dkv_capture_hidden.argtypes = [c_vp, c_vp, c_sz]
lib.dkv_destroy.argtypes = [c_vp]


class ProfEntry(C.Structure):
    _fields_ = [("launches", C.c_int64), ("ms", C.c_double), ("bytes", C.c_double), ("flops", C.c_double)]


# kernel kinds of the profile report; the tile kernels are named as in a rocprofv3 trace, `*` standing for the epilogue
# (0 fp32 product, 1 fused SwiGLU, 2 vocabulary statistics), which the report does not tell apart
PROF_KINDS = ("gemm_dma<*,1,1,1,4,4>", "gemm_dma<*,2,1,1,4,4>", "gemm_dma<*,2,2,2,2,3>", "gemm_dma<*,2,4,2,2,3>",
              "gemm_dma<*,4,4,2,2,2>", "gemm_dma<*,1,3,4,1,4>", "gemm_dma<*,2,3,2,2,3>", "gemm_dma<*,4,3,2,2,2>",
              "gemm_dma<*,3,4,2,2,2>", "gemm_reg",
              "gemm_simt",
              "attention")
GEMM_KINDS = {"dma_32x128": 0, "dma_64x128": 1, "dma_128x128": 2, "dma_128x256": 3, "dma_256x256": 4,
              "dma_128x96": 5, "dma_128x192": 6, "dma_256x192": 7, "dma_192x256": 8, "reg_64x128": 9, "simt": 10}
lib.dkv_profile_begin.argtypes = [c_vp]
lib.dkv_profile_end.argtypes = [c_vp, C.POINTER(ProfEntry)]
lib.dkv_attn_update_workspace_bytes.restype = c_sz
lib.dkv_attn_update_workspace_bytes.argtypes = [c_i32] * 7
lib.dkv_attn_update.argtypes = [c_vp] * 8 + [c_i32] * 8 + [c_vp, c_sz, c_vp]
lib.dkv_attn_update_static.argtypes = [c_vp] * 8 + [c_i32] * 8 + [c_vp]
STATIC_SCRATCH_BYTES = 4 << 20
lib.dkv_concat_reorder.argtypes = [c_vp] * 7 + [c_i32] * 6 + [c_vp]
lib.dkv_peak_copy.argtypes = [c_vp, c_vp, c_sz, c_vp]
lib.dkv_peak_read.argtypes = [c_vp, c_vp, c_sz, c_vp]
lib.dkv_peak_mfma.argtypes = [c_vp, c_i32, C.POINTER(C.c_double), c_vp]
lib.dkv_gemm_workspace_bytes.restype = c_sz
lib.dkv_gemm_workspace_bytes.argtypes = [c_i32] * 4
lib.dkv_gemm.argtypes = [c_vp, c_vp, c_vp, c_i32, c_i32, c_i32, c_i32, c_vp, c_sz, c_vp]
lib.dkv_gemm_with.argtypes = [c_vp, c_vp, c_vp, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32, c_i32, c_vp, c_sz, c_vp]


class DkvError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"dkv error {code}: {text}")
        self.code = code


def last_error():
    return lib.dkv_last_error().decode()


def _check(rc):
    if rc != 0:
        raise DkvError(rc, last_error())


def _ptr(t):
    return None if t is None else c_vp(t.data_ptr())


def _stream():
    return c_vp(torch.cuda.current_stream().cuda_stream)


def _tdtype(dtype):
    return torch.bfloat16 if dtype == BF16 else torch.float32


def model_desc(m):
    return ModelDesc(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn, m.vocab, m.mask_id,
                     m.dtype, m.rms_eps, m.rope_theta)


def run_desc(r, order_ptr=None):
    return RunDesc(r.batch, r.prompt_len, r.gen_len, r.steps, r.block_len, r.refresh_interval, r.variant, r.delay,
                   r.window, r.window_center, r.include_prev, r.remask, getattr(r, "shift_logits", 0), order_ptr)


def upload_weights(model, synth, device="cuda", layers=None):
    """Device tensors in the layouts the library documents, from a dkv_inputs.SynthWeights."""
    td = _tdtype(model.dtype)

    def dev(x, dt=td):
        return torch.from_numpy(np.ascontiguousarray(x)).to(device=device, dtype=dt)

    out = {"embed": dev(synth.embed()), "lm_head": dev(synth.lm_head()),
           "final_norm": dev(synth.final_norm(), torch.float32),
           "wqkv": [], "wo": [], "w_gate_up": [], "w_down": [], "norm1": [], "norm2": []}
    for l in (range(model.n_layers) if layers is None else layers):
        w = synth.layer(l)
        out["wqkv"].append(dev(np.concatenate([w["wq"], w["wk"], w["wv"]], axis=0)))
        out["wo"].append(dev(w["wo"]))
        gu = np.stack([w["w_gate"], w["w_up"]], axis=1).reshape(2 * model.d_ffn, model.d_model)
        out["w_gate_up"].append(dev(gu))
        out["w_down"].append(dev(w["w_down"]))
        out["norm1"].append(dev(w["norm1"], torch.float32))
        out["norm2"].append(dev(w["norm2"], torch.float32))
    return out


def random_weights(model, seed, device="cuda"):
    """Device-side N(0, 0.02) weights of the documented shapes (for throughput runs)."""
    g = torch.Generator(device=device).manual_seed(seed)
    td = _tdtype(model.dtype)

    def mat(r, c):
        return (torch.randn(r, c, generator=g, device=device, dtype=torch.float32) * 0.02).to(td)

    def gain():
        return 1.0 + 0.1 * torch.randn(model.d_model, generator=g, device=device, dtype=torch.float32)

    m = model
    out = {"embed": mat(m.vocab, m.d_model), "lm_head": mat(m.vocab, m.d_model), "final_norm": gain(),
           "wqkv": [], "wo": [], "w_gate_up": [], "w_down": [], "norm1": [], "norm2": []}
    for _ in range(m.n_layers):
        out["wqkv"].append(mat(m.qkv_rows, m.d_model))
        out["wo"].append(mat(m.d_model, m.n_q_heads * m.head_dim))
        out["w_gate_up"].append(mat(2 * m.d_ffn, m.d_model))
        out["w_down"].append(mat(m.d_model, m.d_ffn))
        out["norm1"].append(gain())
        out["norm2"].append(gain())
    return out


class DkvRun:
    """One generation run: owns the device buffers (torch tensors) and the library context."""

    def __init__(self, model, run, weights, prompt, order=None, device="cuda"):
        self.model, self.run, self.w = model, run, weights
        B, L = run.batch, run.seq_len
        self.k = run.k_per_step
        td = _tdtype(model.dtype)
        self.md = model_desc(model)
        self.order = None if order is None else torch.as_tensor(np.asarray(order), dtype=torch.int32, device=device).contiguous()
        self.rd = run_desc(run, _ptr(self.order))
        ws_bytes = lib.dkv_workspace_bytes(C.byref(self.md), C.byref(self.rd))
        if ws_bytes == 0:
            raise DkvError(-1, "descriptors rejected by dkv_workspace_bytes")
        cache_shape = (model.n_layers, B, model.n_kv_heads, L, model.head_dim)
        self.k_cache = torch.empty(cache_shape, dtype=td, device=device)
        self.v_cache = torch.empty(cache_shape, dtype=td, device=device)
        self.tokens = torch.zeros((B, L), dtype=torch.int32, device=device)
        self.tokens[:, :run.prompt_len] = torch.as_tensor(np.asarray(prompt), dtype=torch.int32, device=device)
        self.masked = torch.empty((B, L), dtype=torch.uint8, device=device)
        self.stamp = torch.empty((B, L), dtype=torch.int32, device=device)
        self.decoded_pos = torch.empty((run.steps, B, self.k), dtype=torch.int32, device=device)
        self.decoded_tok = torch.empty((run.steps, B, self.k), dtype=torch.int32, device=device)
        self.decoded_conf = torch.empty((run.steps, B, self.k), dtype=torch.float32, device=device)
        self.workspace = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=device)
        ws_ptr = (self.workspace.data_ptr() + 255) // 256 * 256
        self._arrs = {}
        self._wd = Weights(_ptr(weights["embed"]), _ptr(weights["lm_head"]), _ptr(weights["final_norm"]))
        for name in ("wqkv", "wo", "w_gate_up", "w_down", "norm1", "norm2"):
            arr = (c_vp * model.n_layers)(*[t.data_ptr() for t in weights[name]])
            self._arrs[name] = arr
            setattr(self._wd, name, arr)
        self._bd = Buffers(_ptr(self.k_cache), _ptr(self.v_cache), _ptr(self.tokens), _ptr(self.masked),
                           _ptr(self.stamp), _ptr(self.decoded_pos), _ptr(self.decoded_tok),
                           _ptr(self.decoded_conf), c_vp(ws_ptr), ws_bytes)
        self.ctx = c_vp()
        self.workspace_bytes = ws_bytes
        self._init()

    def _init(self):
        _check(lib.dkv_init_cache(C.byref(self.ctx), C.byref(self.md), C.byref(self._wd), C.byref(self.rd),
                                  C.byref(self._bd), _stream()))

    def reset(self):
        """Start the run again on the same buffers (the prompt part of `tokens` is kept)."""
        self.close()
        self._init()

    def generate(self, steps=None):
        """Enqueue all denoising steps; no host synchronisation in between."""
        for t in range(self.run.steps if steps is None else steps):
            _check(lib.dkv_denoise_step(self.ctx, t, None, None, None))

    def profile_begin(self):
        _check(lib.dkv_profile_begin(self.ctx))

    def profile_end(self):
        arr = (ProfEntry * len(PROF_KINDS))()
        _check(lib.dkv_profile_end(self.ctx, arr))
        return {PROF_KINDS[i]: {"launches": arr[i].launches, "ms": arr[i].ms, "bytes": arr[i].bytes,
                                "flops": arr[i].flops} for i in range(len(PROF_KINDS))}

    def select_active(self, step, active_idx=None, active_off=None):
        ub = c_i32(0)
        _check(lib.dkv_select_active(self.ctx, step, _ptr(active_idx), _ptr(active_off), C.byref(ub)))
        return ub.value

    def denoise_step(self, step, forced_pos=None, forced_tok=None, logits_out=None):
        _check(lib.dkv_denoise_step(self.ctx, step, _ptr(forced_pos), _ptr(forced_tok), _ptr(logits_out)))

    def refresh(self, scope):
        _check(lib.dkv_refresh(self.ctx, scope))

    def read_rows(self):
        cap = self.run.batch * self.run.seq_len
        pos = np.empty(cap, dtype=np.int32)
        off = np.empty(self.run.batch + 1, dtype=np.int32)
        n = c_i32(0)
        _check(lib.dkv_read_rows(self.ctx, pos.ctypes.data, off.ctypes.data, cap, C.byref(n)))
        return pos[:n.value].copy(), off

    def read_candidates(self):
        cap = self.run.batch * self.run.block_len
        pos = np.empty(cap, dtype=np.int32)
        tok = np.empty(cap, dtype=np.int32)
        conf = np.empty(cap, dtype=np.float32)
        off = np.empty(self.run.batch + 1, dtype=np.int32)
        n = c_i32(0)
        _check(lib.dkv_read_candidates(self.ctx, pos.ctypes.data, tok.ctypes.data, conf.ctypes.data,
                                       off.ctypes.data, cap, C.byref(n)))
        return pos[:n.value].copy(), tok[:n.value].copy(), conf[:n.value].copy(), off

    def read_hidden(self, layer=None):
        """Residual stream of the last step at a layer boundary (default: after the last block)."""
        cap = self.run.batch * self.run.seq_len
        out = np.empty((cap, self.model.d_model), dtype=np.float32)
        n = c_i32(0)
        _check(lib.dkv_read_hidden(self.ctx, self.model.n_layers if layer is None else layer, out.ctypes.data,
                                   cap, C.byref(n)))
        return out[:n.value].copy()

    def capture_hidden(self, on=True):
        """Keep the residual stream at every layer boundary of the following steps (device buffer held here)."""
        if on:
            n = (self.model.n_layers + 1) * self.run.batch * self.run.seq_len * self.model.d_model
            self._capture = torch.empty(n, dtype=torch.float32, device=self.k_cache.device)
            _check(lib.dkv_capture_hidden(self.ctx, _ptr(self._capture), n * 4))
        else:
            _check(lib.dkv_capture_hidden(self.ctx, None, 0))
            self._capture = None

    def close(self):
        if self.ctx:
            lib.dkv_destroy(self.ctx)
            self.ctx = c_vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def attn_update_workspace_bytes(batch, n_q_heads, n_kv_heads, seq_len, head_dim, dtype, max_rows_per_seq):
    return lib.dkv_attn_update_workspace_bytes(batch, n_q_heads, n_kv_heads, seq_len, head_dim, dtype,
                                               max_rows_per_seq)


def attn_update(k_cache, v_cache, q, k_new, v_new, active_idx, active_off, out, rows, max_rows_per_seq, dtype,
                workspace):
    B, Hkv, L, dh = k_cache.shape
    Hq = q.shape[1] if q is not None and q.dim() == 3 else out.shape[1]
    _check(lib.dkv_attn_update(_ptr(k_cache), _ptr(v_cache), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(active_idx),
                               _ptr(active_off), _ptr(out), rows, max_rows_per_seq, B, Hq, Hkv, L, dh, dtype,
                               _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
                               _stream()))


def attn_update_static(k_cache, v_cache, q, k_new, v_new, active_idx, active_off, out, rows, max_rows_per_seq,
                       dtype):
    """dkv_attn_update without a workspace argument: the library's static scratch array is used."""
    B, Hkv, L, dh = k_cache.shape
    Hq = q.shape[1] if q is not None and q.dim() == 3 else out.shape[1]
    _check(lib.dkv_attn_update_static(_ptr(k_cache), _ptr(v_cache), _ptr(q), _ptr(k_new), _ptr(v_new),
                                      _ptr(active_idx), _ptr(active_off), _ptr(out), rows, max_rows_per_seq, B, Hq,
                                      Hkv, L, dh, dtype, _stream()))


def concat_reorder(k_cached, v_cached, k_new, v_new, take, dtype):
    """The compact-layout cache operator of Appendix A: gather of concat(cached, new) rows by `take`."""
    B, H, n_c, dh = k_cached.shape
    n_n = k_new.shape[2]
    k_out = torch.empty((B, H, n_c + n_n, dh), dtype=k_cached.dtype, device=k_cached.device)
    v_out = torch.empty_like(k_out)
    _check(lib.dkv_concat_reorder(_ptr(k_cached), _ptr(v_cached), _ptr(k_new), _ptr(v_new), _ptr(take), _ptr(k_out),
                                  _ptr(v_out), B, H, n_c, n_n, dh, dtype, _stream()))
    return k_out, v_out


GEMM_OPT_STAGGER, GEMM_OPT_XCD_GROUP, GEMM_OPT_SWIGLU, GEMM_OPT_STREAM_W = 1, 2, 4, 8


def gemm(x, w, dtype, kind=None, split_k=1, options=0):
    """y = x @ w.T in fp32 through the library's projection kernel (heuristic choice unless `kind`)."""
    m, k = x.shape
    n = w.shape[0]
    if options & GEMM_OPT_SWIGLU:          # fused epilogue: [m, n/2] in the input dtype
        y = torch.empty((m, n // 2), dtype=x.dtype, device=x.device)
    else:
        y = torch.empty((m, n), dtype=torch.float32, device=x.device)
    if kind is None:
        nb = lib.dkv_gemm_workspace_bytes(m, n, k, dtype)
        ws = torch.empty(max(nb, 4), dtype=torch.uint8, device=x.device)
        _check(lib.dkv_gemm(_ptr(x), _ptr(w), _ptr(y), m, n, k, dtype, _ptr(ws), nb, _stream()))
    else:
        slots = 2 if split_k < 0 else split_k          # split_k = -1: the 3/4-share mode, two partial slots
        nb = slots * m * n * 4 if slots > 1 else 0
        ws = torch.empty(max(nb, 4), dtype=torch.uint8, device=x.device)
        _check(lib.dkv_gemm_with(_ptr(x), _ptr(w), _ptr(y), m, n, k, dtype, GEMM_KINDS[kind], split_k, options,
                                 _ptr(ws), nb, _stream()))
    return y


def measured_peaks(reps=5):
    """What this chip sustains on the library's yardstick kernels: cold streaming read and plain copy over 2 GiB
    buffers (larger than the last-level cache), and a register-only dense bf16 MFMA loop.
    Returns {"hbm_read_GBps", "hbm_copy_GBps" (read + written bytes), "mfma_bf16_TFLOPs"}."""
    n = 1 << 31
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1 << 21, dtype=torch.uint8, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    t_read = timed(lambda: _check(lib.dkv_peak_read(_ptr(src), _ptr(sink), n, _stream())))
    t_copy = timed(lambda: _check(lib.dkv_peak_copy(_ptr(src), _ptr(dst), n, _stream())))
    flops = C.c_double(0.0)
    t_mfma = timed(lambda: _check(lib.dkv_peak_mfma(_ptr(sink), 20000, C.byref(flops), _stream())))
    return {"hbm_read_GBps": round(n / t_read * 1e-9, 1), "hbm_copy_GBps": round(2 * n / t_copy * 1e-9, 1),
            "mfma_bf16_TFLOPs": round(flops.value / t_mfma * 1e-12, 1)}
