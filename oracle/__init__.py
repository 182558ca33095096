"""CPU oracle (test infrastructure only; never imported by the product path)."""
from .ckv_oracle import (  # noqa: F401
    TAU, round_to_storage, chunk_bounds, alternating_partition, cosine_similarity, match,
    merge_count, select, select_global, merge, csm_round, clusterable_range, direct_schedule, round_lengths, compress, app_attn,
    annealed_ratio, rounds_to_budget, alg1_decode,
)
