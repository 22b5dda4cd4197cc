"""Seeded synthetic workloads (input generation only; no method arithmetic)."""
from .synth import (WORKLOADS, Workload, peaked, scaled_down, make_chunk, make_chunk_sliced, make_document, gen_tensor,
                    heavy_mask, key_multiplier, CACHE_INSTR, CACHE_SHARED, CACHE_DUAL,
                    SELECT_PER_KV_HEAD, SELECT_PER_LAYER)
