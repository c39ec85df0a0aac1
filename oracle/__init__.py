"""CPU oracle (test infrastructure).  See asyncspade_oracle.c for what it computes.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product path never does.
"""
from .binding import (build, predict_query, ridge_weights, score_keys, topk_select,
                      sparse_decode_attn, select_step, set_threads, f64_to_bf16, overlap_ratio, kv_append,
                      window_push, gather_kv)

__all__ = ["build", "predict_query", "ridge_weights", "score_keys", "topk_select",
           "sparse_decode_attn", "select_step", "set_threads", "f64_to_bf16", "overlap_ratio", "kv_append", "window_push",
           "gather_kv"]
