"""Writes tests/golden/oracle_small_case.txt: router scores, decisions and a few
hidden-state values of a small seeded case, as computed by the CPU oracle.

Calls only `oracle/` and the seeded input recipes.  The paper prints no numeric
example of a forward pass, so this file pins the oracle against drift (an
unintended change to its arithmetic), not against the paper; what pins it to the
mathematics is tests/test_oracle_pins.py.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
sys.path.insert(0, os.path.dirname(HERE))

import workloads as W                      # noqa: E402
from helpers import oracle_model, oracle_params, oracle_pools   # noqa: E402
from oracle import arb_oracle as O         # noqa: E402

MODEL = W.ModelShape("golden-small", 2, 64, 4, 2, 16, 96, 211, kv_block=4)
WORK = W.Workload("golden-small", MODEL, 3, (6, 19), ("uniform", 1, 7), "shuffled", "prefill", 0.0,
                  ("const", 0.5), 41)


def compute():
    batch = W.make_batch(WORK)
    weights = W.make_weights(MODEL, WORK.seed, sigma=0.2, gain_jitter=0.1, b_head=0.03125)
    m, p = oracle_model(MODEL), oracle_params(weights)
    kp, vp = oracle_pools(*W.make_kv_pools(WORK, batch))
    cu_p = np.concatenate([[0], np.cumsum(batch.prefix_lens)]).astype(np.int32)
    O.prefill(m, p, kp, vp, W.prompt_token_ids(WORK, batch), cu_p, batch.block_tables)
    scores, esc, y = O.score_steps(m, p, kp, vp, batch.token_ids, batch.prefix_lens, batch.cu_step_lens,
                                   batch.block_tables, batch.tau)
    return batch, scores, esc, y


if __name__ == "__main__":
    batch, scores, esc, y = compute()
    with open(os.path.join(HERE, "oracle_small_case.txt"), "w") as f:
        f.write("# written by tests/golden/make_golden.py from oracle/arb_oracle.py (no paper value exists)\n")
        f.write("prefix_lens " + " ".join(map(str, batch.prefix_lens)) + "\n")
        f.write("step_lens " + " ".join(map(str, batch.step_lens)) + "\n")
        f.write("scores " + " ".join(f"{v:.12e}" for v in scores) + "\n")
        f.write("escalate " + " ".join(map(str, esc)) + "\n")
        f.write("hidden_first_row_head " + " ".join(f"{v:.12e}" for v in y[0, :4]) + "\n")
        f.write("hidden_last_row_tail " + " ".join(f"{v:.12e}" for v in y[-1, -4:]) + "\n")
