"""Seeded synthetic workloads shared by the CPU checks and the GPU path."""
from .configs import (ALL, C1, C2, C3, C4, C5, ROUTER_1P5B, TARGET_8B, TINY, ModelShape, Workload,  # noqa: F401
                      scaled)
from .generate import (Batch, Weights, bf16_bits, kv_pool_blocks, kv_pool_shape, make_batch,  # noqa: F401
                       make_kv_pools, make_weights, normal_bf16, normal_bf16_at, prompt_token_ids,
                       uniform_ints)
