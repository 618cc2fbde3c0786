"""The entry point that allocates nothing (arb_score_steps_noalloc: workspace in a static device
array) against arb_score_steps with a caller workspace: same kernels, so the same bits; two calls
in a row, the second on a smaller batch, so that the array still holds the first call's contents."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2512_05033_amd as A
    A.load_library()
    return A


def _both(A, sess, dbatch, B, T):
    """One call of each entry point on the same inputs -> ((scores, escalate, hidden), (same)), all on the host."""
    import harness  # noqa: F401
    d = sess.workload.model.d_model
    out = []
    for noalloc in (False, True):
        scores = torch.full((B,), float("nan"), device="cuda")
        esc = torch.full((B,), 7, dtype=torch.uint8, device="cuda")
        hidden = torch.zeros(T, d, dtype=torch.bfloat16, device="cuda")
        if noalloc:
            A.arb_score_steps_noalloc(sess.model, sess.kv, dbatch, sess.batch.tau, scores=scores, escalate=esc, hidden=hidden)
        else:
            A.arb_score_steps(sess.model, sess.kv, dbatch, sess.batch.tau, ws=sess.ws, scores=scores, escalate=esc, hidden=hidden)
        torch.cuda.synchronize()
        out.append((scores.cpu().numpy(), esc.cpu().numpy(), W.bf16_bits(hidden)))
    return out


@pytest.mark.parametrize("w", [W.scaled(W.C1, batch=4), W.scaled(W.C2, n_layers=2, batch=2)], ids=["tiny", "router-shape"])
def test_noalloc_matches_the_workspace_entry_point_twice_in_a_row(A, w):
    import harness
    sess = harness.setup(w, "cuda", gain_jitter=0.1)
    batch = sess.batch
    ref, got = _both(A, sess, sess.dbatch, batch.batch, batch.total_tokens)
    assert np.isfinite(ref[0]).all() and set(np.unique(ref[1])) <= {0, 1}
    for r, g in zip(ref, got):
        assert np.array_equal(r, g)
    # a smaller batch next: the last sequence alone, then the first two with shorter steps
    for rows in ([batch.batch - 1], [0, 1]):
        sub = batch.select(rows)
        if len(rows) == 2:
            keep = np.maximum(sub.step_lens // 2, 1)
            tok = np.concatenate([sub.token_ids[sub.cu_step_lens[i]:sub.cu_step_lens[i] + keep[i]] for i in range(2)])
            sub = W.Batch(sub.prefix_lens, np.concatenate([[0], np.cumsum(keep)]).astype(np.int32), sub.block_tables,
                          tok.astype(np.int32), sub.n_blocks, sub.kv_block, sub.tau, sub.spare_blocks)
        ref, got = _both(A, sess, harness.device_batch(sub), sub.batch, sub.total_tokens)
        for r, g in zip(ref, got):
            assert np.array_equal(r, g)


def test_noalloc_rejects_what_does_not_fit(A):
    """The full 1.5B-router batch (1024 step tokens) needs more than the static array holds."""
    import harness
    w = W.scaled(W.C2, n_layers=1)
    sess = harness.setup(w, "cuda")
    need = sess.model.workspace_bytes(sess.batch.batch, sess.batch.total_tokens, sess.dbatch.max_ctx)
    assert need > A.NOALLOC_SCRATCH_BYTES
    B, T = sess.batch.batch, sess.batch.total_tokens
    scores = torch.zeros(B, device="cuda"); esc = torch.zeros(B, dtype=torch.uint8, device="cuda")
    with pytest.raises(A.ArbError) as e:
        A.arb_score_steps_noalloc(sess.model, sess.kv, sess.dbatch, 0.0, scores=scores, escalate=esc)
    assert e.value.status == A.ARB_ECAPACITY and "ARB_NOALLOC_SCRATCH_BYTES" in str(e.value)
    torch.cuda.synchronize()
