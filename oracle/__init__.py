"""fp64 CPU oracle of the Judge Q eviction path -- test infrastructure, never a product path."""
from .jq_oracle import (  # noqa: F401
    build, compact, evict, evict_batch, hit_rate, map_mse, num_threads, pool, score, score_lse, score_tail, score_window, select_topk, stream_step,
)
