"""Seeded token, order and microbenchmark inputs."""
from dataclasses import dataclass
import numpy as np
from .configs import BF16, FP32
from .rng import normal_f32, uniform_ids, permutation, _gen


def prompt_tokens(model, run, seed):
    """[batch, prompt_len] ids uniform on [0, vocab) excluding the MASK id."""
    ids = uniform_ids(seed, 0, (run.batch, run.prompt_len), 0, model.vocab - 1)
    # ids >= mask_id shift up by one so MASK never appears (mask_id = vocab-1 leaves them as is)
    return np.where(ids >= model.mask_id, ids + 1, ids).astype(np.int32)


def random_block_order(run, seed):
    """[batch, gen_len] decode order: each block's positions shuffled, blocks left to right.

    Entries are absolute sequence positions (prompt_len + offset)."""
    out = np.empty((run.batch, run.gen_len), dtype=np.int32)
    for b in range(run.batch):
        for j in range(run.n_blocks):
            lo = j * run.block_len
            p = permutation(seed, b * 4096 + j, run.block_len)
            out[b, lo:lo + run.block_len] = run.prompt_len + lo + p
    return out


@dataclass(frozen=True)
class AttnUpdateShape:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    seq_len: int
    head_dim: int
    dtype: int = BF16


CONFIG1_SHAPE = AttnUpdateShape(batch=8, n_q_heads=32, n_kv_heads=32, seq_len=1024, head_dim=128)
CONFIG1_ACTIVE_SIZES = (1, 8, 32, 128, 512)


def attn_update_case(shape, n_active, seed, ragged=None):
    """Inputs of one scatter-then-attend call.

    Returns dict with
      k_cache, v_cache [B, Hkv, L, dh]   q [R, Hq, dh]   k_new, v_new [R, Hkv, dh]
      active_idx [R] (positions, sorted per sequence)   active_off [B+1]
    all ~N(0,1) (rounded to bfloat16 values when shape.dtype is BF16).
    `ragged`, if given, lists a per-sequence active count instead of `n_active`."""
    B, L = shape.batch, shape.seq_len
    counts = list(ragged) if ragged is not None else [n_active] * B
    assert len(counts) == B and all(0 <= c <= L for c in counts)
    off = np.zeros(B + 1, dtype=np.int32)
    off[1:] = np.cumsum(counts)
    R = int(off[-1])
    idx = np.empty(R, dtype=np.int32)
    for b in range(B):
        idx[off[b]:off[b + 1]] = np.sort(permutation(seed, 10 + b, L)[:counts[b]])
    bf = shape.dtype == BF16
    dh = shape.head_dim
    return {
        "k_cache": normal_f32(seed, 1, (B, shape.n_kv_heads, L, dh), bf16=bf),
        "v_cache": normal_f32(seed, 2, (B, shape.n_kv_heads, L, dh), bf16=bf),
        "q": normal_f32(seed, 3, (R, shape.n_q_heads, dh), bf16=bf),
        "k_new": normal_f32(seed, 4, (R, shape.n_kv_heads, dh), bf16=bf),
        "v_new": normal_f32(seed, 5, (R, shape.n_kv_heads, dh), bf16=bf),
        "active_idx": idx,
        "active_off": off,
    }
