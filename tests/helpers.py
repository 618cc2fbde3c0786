"""Glue between the seeded workloads and the oracle's plain-array interface."""
from __future__ import annotations

import numpy as np

import workloads as W
from oracle import arb_oracle as O


# Hidden-state bars (max|got - ref| / max|ref| over the output tensor).  2e-2 is the stated bar.  A deep model
# with random weights amplifies perturbations: rounding nothing but the operands of the matrix products to bf16
# (inside otherwise exact fp64 arithmetic: forward_bf16_operands below, built from the oracle's own functions)
# already moves the output of the 28-layer 1.5B-class shape by 2e-2 to 2.7e-2, depending on the sample.  So an
# end-to-end run at full depth measures that floor on its own sample and is held to
# max(2e-2, FLOOR_FACTOR x floor); every layer is also checked on its own, from the oracle's residual stream,
# against the stated 2e-2.
HIDDEN_TOL, SCORE_TOL, FLOOR_FACTOR = 2e-2, 1e-2, 1.3


def round_bf16(x: np.ndarray) -> np.ndarray:
    return O.bf16_to_float(O.float_to_bf16(x))


def forward_bf16_operands(m: O.Model, p: O.Params, kp, vp, token_ids, prefix_lens, cu_step_lens, block_tables,
                          rnd, depths, progress=None):
    """The oracle's forward, stage by stage, with `rnd` applied to the inputs of the matrix products
    (normed activations, rotated queries, attention output, SwiGLU output).  Returns the final-normed
    hidden states after each depth in `depths`.  With rnd = identity it is O.forward (tested)."""
    blk, Hq, Hkv, hd = m.kv_block, m.n_q_heads, m.n_kv_heads, m.head_dim
    pl, cu, bt = prefix_lens, cu_step_lens, block_tables
    pos, slots = O.positions(pl, cu), O.slot_mapping(pl, cu, bt, blk)
    h = O.embed(p.embed, token_ids)
    T, out = h.shape[0], {}
    for l in range(m.n_layers):
        x = rnd(O.rmsnorm(h, p.g_attn[l], m.rms_eps))
        qkv = (x @ O.as_float(p.wqkv[l]).T).reshape(T, Hq + 2 * Hkv, hd)
        q = rnd(O.rope(qkv[:, :Hq], pos, m.rope_base))
        O.kv_append(kp[l], vp[l], slots, O.rope(qkv[:, Hq:Hq + Hkv], pos, m.rope_base), qkv[:, Hq + Hkv:], blk)
        o = rnd(O.append_attention(q, kp[l], vp[l], pl, cu, bt, blk))
        h = h + o.reshape(T, Hq * hd) @ O.as_float(p.wo[l]).T
        gu = rnd(O.rmsnorm(h, p.g_mlp[l], m.rms_eps)) @ O.as_float(p.wgu[l]).T
        F = gu.shape[1] // 2
        h = h + rnd(O.silu(gu[:, :F]) * gu[:, F:]) @ O.as_float(p.wd[l]).T
        if l + 1 in depths:
            out[l + 1] = O.rmsnorm(h, p.g_final, m.rms_eps)
        if progress:
            progress(l + 1)
    return out


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


def rms_err(got: np.ndarray, ref: np.ndarray) -> float:
    """sqrt(mean (got - ref)^2 / mean ref^2)."""
    return float(np.sqrt(np.mean((got.astype(np.float64) - ref) ** 2) / np.mean(ref ** 2)))
