"""Workload descriptors: model shapes, run schedules and the five benchmark configurations.

Pure data. Integer codes match the constants of the C boundary header.
"""
from dataclasses import dataclass, replace

BF16, FP32 = 0, 1
DECODE, GREEDY, PREFILL, PD = 0, 1, 2, 3
CONFIDENCE, RANDOM_ORDER = 0, 1
CENTER_CUR, CENTER_PREV = 0, 1
SCOPE_ALL, SCOPE_GEN = 0, 1


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    mask_id: int
    dtype: int = BF16
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def qkv_rows(self):
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    def with_layers(self, n):
        return replace(self, n_layers=n)


@dataclass(frozen=True)
class RunShape:
    batch: int
    prompt_len: int
    gen_len: int
    steps: int
    block_len: int
    refresh_interval: int
    variant: int = DECODE
    delay: int = 1
    window: int = 0
    window_center: int = CENTER_CUR
    include_prev: int = 1
    remask: int = CONFIDENCE
    shift_logits: int = 0

    @property
    def seq_len(self):
        return self.prompt_len + self.gen_len

    @property
    def n_blocks(self):
        return self.gen_len // self.block_len

    @property
    def steps_per_block(self):
        return self.steps // self.n_blocks

    @property
    def k_per_step(self):
        return self.block_len // self.steps_per_block


TINY = ModelShape(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=4, head_dim=32, d_ffn=512,
                  vocab=1024, mask_id=1023, dtype=FP32)
LLADA_8B = ModelShape(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=32, head_dim=128,
                      d_ffn=12288, vocab=126464, mask_id=126463, dtype=BF16)
DREAM_7B = ModelShape(n_layers=28, d_model=3584, n_q_heads=28, n_kv_heads=4, head_dim=128,
                      d_ffn=18944, vocab=152064, mask_id=152063, dtype=BF16)

# index -> (model, run, weight seed, prompt seed, order seed or None)
CONFIGS = {
    0: (TINY, RunShape(batch=1, prompt_len=32, gen_len=32, steps=32, block_len=32,
                       refresh_interval=8, variant=DECODE), 1000, 1001, None),
    2: (LLADA_8B, RunShape(batch=1, prompt_len=256, gen_len=256, steps=256, block_len=32,
                           refresh_interval=8, variant=DECODE), 1200, 1201, None),
    3: (LLADA_8B, RunShape(batch=4, prompt_len=1024, gen_len=512, steps=512, block_len=64,
                           refresh_interval=4, variant=GREEDY, window=4, window_center=CENTER_CUR,
                           include_prev=1, remask=RANDOM_ORDER), 1300, 1301, 1302),
    4: (DREAM_7B, RunShape(batch=16, prompt_len=512, gen_len=256, steps=256, block_len=256,
                           refresh_interval=4, variant=PD), 1400, 1401, None),
}


def model_run(index):
    """(model, run, weight_seed, prompt_seed, order_seed) of a full-model configuration."""
    return CONFIGS[index]
