"""Glue between the seeded workloads and the oracle's plain-array interface."""
from __future__ import annotations

import numpy as np

import workloads as W
from oracle import arb_oracle as O


# Hidden-state bars (max|got - ref| / max|ref| over the output tensor).  2e-2 is the stated bar.  At the full
# 28-layer depth of the 1.5B-class shape, rounding nothing but the operands of the matrix products to bf16
# (inside otherwise exact fp64 arithmetic) already moves the output by 2e-2 to 2.7e-2, depending on the
# sample (test_bf16_floor.py), so end-to-end runs that deep are held to 4e-2 and every layer is checked on
# its own, from the oracle's residual stream, against the 2e-2 bar.
HIDDEN_TOL, FULL_DEPTH_HIDDEN_TOL, SCORE_TOL = 2e-2, 4e-2, 1e-2


def oracle_model(m: W.ModelShape) -> O.Model:
    return O.Model(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn, m.vocab,
                   m.rms_eps, m.rope_base, m.kv_block)


def oracle_params(w: W.Weights) -> O.Params:
    bits = W.bf16_bits
    f32 = lambda t: t.detach().cpu().numpy().astype(np.float64)
    return O.Params(embed=bits(w.embed), wqkv=[bits(t) for t in w.wqkv], wo=[bits(t) for t in w.wo],
                    wgu=[bits(t) for t in w.wgu], wd=[bits(t) for t in w.wd],
                    g_attn=[f32(t) for t in w.g_attn], g_mlp=[f32(t) for t in w.g_mlp],
                    g_final=f32(w.g_final), w_head=f32(w.w_head), b_head=w.b_head)


def oracle_pools(ks, vs):
    return [W.bf16_bits(k).copy() for k in ks], [W.bf16_bits(v).copy() for v in vs]


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max|got - ref| / max|ref| over the tensor."""
    return float(np.max(np.abs(got.astype(np.float64) - ref)) / np.max(np.abs(ref)))
