"""Random-init transformer weights, produced tensor by tensor from a seed.

Layouts (all row-major, y = a @ W.T so every matrix is [out_features, in_features]):
  embed    [vocab, d_model]          lm_head [vocab, d_model]
  wq [Hq*dh, d]  wk [Hkv*dh, d]  wv [Hkv*dh, d]   (head-major rows)
  wo [d, Hq*dh]  w_gate [F, d]  w_up [F, d]  w_down [d, F]
  norm1, norm2, final_norm [d]  (float32 gains drawn around 1 so a dropped gain is visible)
Matrix entries are N(0, 0.02); in a bf16 model they are rounded to bfloat16 values
(held as float32), so both consumers start from exactly representable numbers.
"""
import numpy as np
from .configs import BF16
from .rng import normal_f32

_STD = 0.02
_GAIN_STD = 0.1
# stream ids of the per-layer tensors
_WQ, _WK, _WV, _WO, _WG, _WU, _WD, _N1, _N2 = range(9)
_EMBED, _HEAD, _FNORM = 1_000_001, 1_000_002, 1_000_003


class SynthWeights:
    def __init__(self, model, seed, cache_layers=True, hold_float64=False):
        """hold_float64: keep the matrices widened to float64 (same values; a consumer that computes in
        float64 then does not widen 10^8 entries on every use)."""
        self.model = model
        self.seed = seed
        self._bf16 = model.dtype == BF16
        self._cache = {} if cache_layers else None
        self._f64 = hold_float64

    def _mat(self, stream, shape):
        m = normal_f32(self.seed, stream, shape, std=_STD, bf16=self._bf16)
        return m.astype(np.float64) if self._f64 else m

    def _gain(self, stream):
        return normal_f32(self.seed, stream, (self.model.d_model,), std=_GAIN_STD, mean=1.0)

    def embed(self):
        return self._memo("embed", lambda: self._mat(_EMBED, (self.model.vocab, self.model.d_model)))

    def lm_head(self):
        return self._memo("head", lambda: self._mat(_HEAD, (self.model.vocab, self.model.d_model)))

    def final_norm(self):
        return self._memo("fnorm", lambda: self._gain(_FNORM))

    def layer(self, l):
        return self._memo(("layer", l), lambda: self._layer(l))

    def _layer(self, l):
        m = self.model
        s = 100 + 16 * l
        d, dh, F = m.d_model, m.head_dim, m.d_ffn
        return {
            "wq": self._mat(s + _WQ, (m.n_q_heads * dh, d)),
            "wk": self._mat(s + _WK, (m.n_kv_heads * dh, d)),
            "wv": self._mat(s + _WV, (m.n_kv_heads * dh, d)),
            "wo": self._mat(s + _WO, (d, m.n_q_heads * dh)),
            "w_gate": self._mat(s + _WG, (F, d)),
            "w_up": self._mat(s + _WU, (F, d)),
            "w_down": self._mat(s + _WD, (d, F)),
            "norm1": self._gain(s + _N1),
            "norm2": self._gain(s + _N2),
        }

    def _memo(self, key, fn):
        if self._cache is None:
            return fn()
        if key not in self._cache:
            self._cache[key] = fn()
        return self._cache[key]
