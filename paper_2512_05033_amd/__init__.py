"""MI355X-native step-scoring forward and routing decision of Arbitrage.

The compute lives in libarb.so (HIP, gfx950; sources in csrc/, C ABI in
include/arb.h); this package is the thin binding over it.
"""
from .binding import (ARB_ACCEPT_IF_GT, ARB_ECAPACITY, ARB_EHIP, ARB_EINVAL, ARB_EPI_RESIDUAL_F32,  # noqa: F401
                      ARB_EPI_STORE_BF16, ARB_EPI_STORE_F32, ARB_EPI_SWIGLU_BF16, ARB_ESCALATE_IF_GT, ARB_ESHAPE, ARB_EUNSUPPORTED,
                      ARB_OK, ARB_POOL_LAST, ARB_HEAD_NONE, ARB_HEAD_LINEAR, ARB_HEAD_TWO_CLASS, ARB_POOL_MEAN, ARB_STAGE_ATTENTION, ARB_STAGE_DOWN,
                      ARB_STAGE_GATE_UP, ARB_STAGE_GATE_UP_LARGE, ARB_STAGE_NORM, ARB_STAGE_OPROJ, ARB_STAGE_QKV, ARB_STAGE_ROPE_APPEND, EXPORTS, NOALLOC_SCRATCH_BYTES,
                      StageTimer, ArbError, DeviceBatch, KVCache, Model, QuantizedWeights,
                      arb_budget_threshold, arb_first_stop, arb_step_advance, arb_pack_steps, arb_gemm_large_tile_columns, arb_next_token, arb_pack_k_blocked, arb_advantage_route, arb_prefill, arb_route, arb_score_steps, arb_score_steps_noalloc, arb_slot_mapping, arb_stage_attention, arb_w4_quantize, arb_w3_quantize,
                      arb_stage_gemm, arb_stage_gemm_w4, arb_stage_layers, arb_stage_norm_pool_head, arb_stage_rmsnorm, arb_stage_rope_append,
                      load_library)
