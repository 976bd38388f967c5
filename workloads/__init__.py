"""Seeded synthetic inputs for the KV-cache hot path (token streams, page tables, KV bytes, index
fillers, op streams). Serves the CPU oracle and the HIP library alike and contains none of the
method's arithmetic: no hashing, no table probing, no page copies."""
from .configs import (Geometry, Workload, make_workload, make_tokens, make_scaled_tokens,
                      filler_keys, fill_pool_numpy, fill_pool_torch, zipf_sample, CONFIG_NAMES)

__all__ = ["Geometry", "Workload", "make_workload", "make_tokens", "make_scaled_tokens",
           "filler_keys", "fill_pool_numpy", "fill_pool_torch", "zipf_sample", "CONFIG_NAMES"]
