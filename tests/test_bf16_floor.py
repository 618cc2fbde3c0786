"""How far bf16 operands alone move the forward: the fp64 oracle's own steps with
only the inputs of the matrix products (normed activations, rotated queries,
attention output, SwiGLU output) rounded to bf16.  This is a property of the
network and of the number format, not of any kernel; end-to-end runs at full
depth measure it on their own sample and are held to a multiple of it
(helpers.FLOOR_FACTOR)."""
from dataclasses import replace

import numpy as np
import pytest

import workloads as W
from helpers import FLOOR_FACTOR, HIDDEN_TOL, forward_bf16_operands, oracle_model, oracle_params, oracle_pools, rel_err, round_bf16
from oracle import arb_oracle as O


@pytest.mark.parametrize("shape,seed,depths", [(W.ROUTER_1P5B, W.C2.seed, (2, 8, 28)),
                                               (W.TARGET_8B, W.C3.seed, (2, 8))])
def test_bf16_operand_rounding_floor(shape, seed, depths):
    shape = replace(shape, n_layers=depths[-1])
    w = W.Workload("floor", shape, 2, (0, 0), ("fixed", 1, 1), "shuffled", "synthetic", 1.0, ("const", 0.0), seed)
    batch = W.make_batch(w, prefix_lens=[96, 200], step_lens=[64, 64])
    m, p = oracle_model(w.model), oracle_params(W.make_weights(w.model, w.seed, "cpu"))
    args = (batch.token_ids, batch.prefix_lens, batch.cu_step_lens, batch.block_tables)
    exact = forward_bf16_operands(m, p, *oracle_pools(*W.make_kv_pools(w, batch, "cpu")), *args, lambda a: a, depths)
    rounded = forward_bf16_operands(m, p, *oracle_pools(*W.make_kv_pools(w, batch, "cpu")), *args, round_bf16, depths)
    floor = {l: rel_err(round_bf16(rounded[l]), exact[l]) for l in depths}
    print("bf16 operand floor by depth:", floor)
    assert floor[depths[0]] < 0.65 * HIDDEN_TOL               # the stated bar has room at small depth,
    assert floor[depths[-1]] > 0.75 * HIDDEN_TOL              # none at the deepest one,
    assert FLOOR_FACTOR * floor[depths[-1]] < 2 * HIDDEN_TOL  # and the full-depth bar stays within twice the stated one
    assert all(floor[a] < floor[b] for a, b in zip(depths, depths[1:]))     # the drift compounds with depth


def test_floor_model_without_rounding_is_the_oracle_forward():
    w = W.scaled(W.C1, batch=2)
    batch = W.make_batch(w)
    m, p = oracle_model(w.model), oracle_params(W.make_weights(w.model, w.seed, "cpu"))
    pools = lambda: oracle_pools(*W.make_kv_pools(w, batch, "cpu"))
    got = forward_bf16_operands(m, p, *pools(), batch.token_ids, batch.prefix_lens, batch.cu_step_lens,
                                batch.block_tables, lambda a: a, (m.n_layers,))[m.n_layers]
    assert np.array_equal(got, O.forward(m, p, *pools(), batch.token_ids, batch.prefix_lens, batch.cu_step_lens,
                                         batch.block_tables))
