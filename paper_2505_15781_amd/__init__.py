"""MI355X-native dKV-Cache hot path (arxiv 2505.15781): HIP library + thin ctypes binding."""
from .binding import (lib, DkvError, DkvRun, attn_update, attn_update_workspace_bytes, gemm, GEMM_KINDS,
                      concat_reorder,
                      BF16, FP32, last_error)
