"""How far bf16 operands alone move the forward: the fp64 oracle's own steps with
only the inputs of the matrix products (normed activations, rotated queries,
attention output, SwiGLU output) rounded to bf16.  This is a property of the
network and of the number format, not of any kernel; it derives the bar that
end-to-end runs at full depth are held to (helpers.FULL_DEPTH_HIDDEN_TOL)."""
from dataclasses import replace

import numpy as np
import pytest

import workloads as W
from helpers import FULL_DEPTH_HIDDEN_TOL, HIDDEN_TOL, oracle_model, oracle_params, oracle_pools, rel_err
from oracle import arb_oracle as O


def _rb(x):
    return O.bf16_to_float(O.float_to_bf16(x))


def _forward(m, p, kp, vp, batch, rnd, depths):
    blk, Hq, Hkv, hd = m.kv_block, m.n_q_heads, m.n_kv_heads, m.head_dim
    pl, cu, bt = batch.prefix_lens, batch.cu_step_lens, batch.block_tables
    pos, slots = O.positions(pl, cu), O.slot_mapping(pl, cu, bt, blk)
    h = O.embed(p.embed, batch.token_ids)
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
    return out


@pytest.mark.parametrize("shape,seed,depths", [(W.ROUTER_1P5B, W.C2.seed, (2, 8, 28)),
                                               (W.TARGET_8B, W.C3.seed, (2, 8))])
def test_bf16_operand_rounding_floor(shape, seed, depths):
    shape = replace(shape, n_layers=depths[-1])
    w = W.Workload("floor", shape, 2, (0, 0), ("fixed", 1, 1), "shuffled", "synthetic", 1.0, ("const", 0.0), seed)
    batch = W.make_batch(w, prefix_lens=[96, 200], step_lens=[64, 64])
    m, p = oracle_model(w.model), oracle_params(W.make_weights(w.model, w.seed, "cpu"))
    exact = _forward(m, p, *oracle_pools(*W.make_kv_pools(w, batch, "cpu")), batch, lambda a: a, depths)
    rounded = _forward(m, p, *oracle_pools(*W.make_kv_pools(w, batch, "cpu")), batch, _rb, depths)
    floor = {l: rel_err(_rb(rounded[l]), exact[l]) for l in depths}
    print("bf16 operand floor by depth:", floor)
    assert floor[depths[0]] < 0.65 * HIDDEN_TOL               # the stated bar has room at small depth,
    assert floor[depths[-1]] > 0.75 * HIDDEN_TOL              # none at the deepest one,
    assert 1.25 * floor[depths[-1]] < FULL_DEPTH_HIDDEN_TOL   # which is what the full-depth bar allows for
    assert all(floor[a] < floor[b] for a, b in zip(depths, depths[1:]))     # the drift compounds with depth


def test_floor_model_without_rounding_is_the_oracle_forward():
    w = W.scaled(W.C1, batch=2)
    batch = W.make_batch(w)
    m, p = oracle_model(w.model), oracle_params(W.make_weights(w.model, w.seed, "cpu"))
    pools = lambda: oracle_pools(*W.make_kv_pools(w, batch, "cpu"))
    got = _forward(m, p, *pools(), batch, lambda a: a, (m.n_layers,))[m.n_layers]
    assert np.array_equal(got, O.forward(m, p, *pools(), batch.token_ids, batch.prefix_lens, batch.cu_step_lens,
                                         batch.block_tables))
