"""CPU oracle (test infrastructure only; never imported by the product path)."""
from .lshmoe_oracle import (  # noqa: F401
    widen, narrow, hash_ref, sphere_hash_ref, gate_logits_ref, combine_codes, group_ref, centroid_ref, restore_ref, restore_backward_ref,
    compress_backward_ref, combine_backward_ref, row_rel_err,
)
