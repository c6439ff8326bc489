"""Counter-based random draws and storage rounding.

Every draw is keyed by (seed, stream, chunk) through a Philox bit generator, so
any tensor (or any row chunk of it) can be produced on its own, in any order,
on any number of threads, and both consumers see identical values.
"""
from concurrent.futures import ThreadPoolExecutor
import os
import numpy as np

_CHUNK_ELEMS = 1 << 20      # draws are keyed per chunk: small enough that every large tensor fills all threads


def _gen(seed, stream, chunk=0):
    return np.random.Generator(np.random.Philox(key=[(int(seed) << 20) ^ int(stream), int(chunk)]))


def bf16_round(x):
    """Round float32 values to the nearest bfloat16 (ties to even), returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x):
    """The 16-bit patterns of values already representable in bfloat16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b):
    """Widen bfloat16 bit patterns (uint16) to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_f32(seed, stream, shape, std=1.0, mean=0.0, bf16=False, threads=None):
    """N(mean, std) draws as float32, optionally rounded to bfloat16 values."""
    n = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(n, dtype=np.float32)
    nchunks = max(1, (n + _CHUNK_ELEMS - 1) // _CHUNK_ELEMS)

    def fill(c):
        lo = c * _CHUNK_ELEMS
        hi = min(n, lo + _CHUNK_ELEMS)
        v = _gen(seed, stream, c).standard_normal(hi - lo, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        if mean != 0.0:
            v += np.float32(mean)
        out[lo:hi] = bf16_round(v) if bf16 else v

    if nchunks == 1:
        fill(0)
    else:
        workers = threads or min(16, os.cpu_count() or 1)
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(fill, range(nchunks)))
    return out.reshape(shape)


def uniform_ids(seed, stream, shape, low, high):
    """Integers uniform on [low, high) as int32."""
    return _gen(seed, stream).integers(low, high, size=shape, dtype=np.int64).astype(np.int32)


def permutation(seed, stream, n):
    """A uniform random permutation of range(n) as int32."""
    return _gen(seed, stream).permutation(n).astype(np.int32)
