"""Seeded synthetic KV-cache inputs.

This package only draws random numbers and shapes them into key / value / query
tensors. It holds none of the compression or attention arithmetic and imports
neither the CPU oracle nor the HIP library, so both sides of a parity test can
be fed from it.
"""
from .kv import (  # noqa: F401
    ar1_keys_host,
    kv_host,
    kv_device,
    query_host,
    head_seed,
    to_storage,
)
