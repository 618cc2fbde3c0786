"""The seeded input recipes: determinism, distribution, and table structure."""
import numpy as np
import torch

import workloads as W
from workloads.generate import _GOLDEN, hash64, stream_key


def test_hash_is_splitmix64():
    # first outputs of splitmix64 seeded with 0 (state advances by the golden gamma):
    # published test vector 0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F
    got = hash64(torch.arange(3, dtype=torch.int64) * _GOLDEN, 0)
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert [int(v) & ((1 << 64) - 1) for v in got] == want


def test_normal_stream_is_deterministic_indexable_and_normal():
    a = W.normal_bf16(5, "w", (1000, 64), 0.02)
    b = W.normal_bf16(5, "w", (1000, 64), 0.02)
    assert torch.equal(a, b)
    idx = torch.tensor([0, 63, 64, 63999], dtype=torch.int64)
    assert torch.equal(W.normal_bf16_at(5, "w", idx, 0.02), a.view(-1)[idx])
    assert not torch.equal(a, W.normal_bf16(6, "w", (1000, 64), 0.02))
    assert stream_key(5, "w") != stream_key(5, "v")
    x = a.double().numpy().ravel() / 0.02
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1) < 0.02
    assert abs(np.mean(np.abs(x) < 1) - 0.6827) < 0.01 and abs(np.mean(np.abs(x) > 2) - 0.0455) < 0.005


def test_token_ids_in_range_and_spread():
    ids = W.uniform_ints(1, "ids", 100000, 32000).numpy()
    assert ids.min() >= 0 and ids.max() < 32000 and len(np.unique(ids)) > 30000


def test_batches_follow_the_recipes():
    for name, w in W.ALL.items():
        b = W.make_batch(w)
        blk = w.model.kv_block
        assert b.batch == w.batch and b.cu_step_lens[0] == 0
        assert b.prefix_lens.min() >= w.prefix[0] and b.prefix_lens.max() <= w.prefix[1]
        need = (b.prefix_lens + b.step_lens + blk - 1) // blk
        used = np.concatenate([b.block_tables[i, :need[i]] for i in range(b.batch)])
        assert len(np.unique(used)) == len(used) == need.sum()            # no block shared
        assert used.min() >= 0 and b.block_tables.max() < b.n_blocks
        assert not set(b.spare_blocks.tolist()) & set(used.tolist())
        assert len(b.token_ids) == b.total_tokens and b.token_ids.max() < w.model.vocab
        if w.tables == "identity":
            assert np.array_equal(used, np.arange(len(used)))
    assert W.make_batch(W.C5).step_lens.tolist() == [1, 64] * 16
    assert W.make_batch(W.C2).total_tokens == 1024 and W.make_batch(W.C3).total_tokens == 512
    c4 = W.make_batch(W.C4)
    assert c4.step_lens.min() >= 16 and c4.step_lens.max() <= 128 and c4.tau != 0.0
    assert c4.tau == W.make_batch(W.C4).tau


def test_pool_blocks_match_full_pool_and_select():
    w = W.scaled(W.C2, n_layers=1, batch=2)
    b = W.make_batch(w)
    ks, vs = W.make_kv_pools(w, b)
    ids = [0, 5, b.n_blocks - 1]
    assert torch.equal(W.kv_pool_blocks(w, 0, "k", ids), ks[0][ids])
    assert torch.equal(W.kv_pool_blocks(w, 0, "v", ids), vs[0][ids])
    sub = b.select([1])
    assert sub.total_tokens == b.step_lens[1] and np.array_equal(sub.block_tables[0], b.block_tables[1])
    assert abs(ks[0].float().std().item() - 0.8) < 0.01


def test_weight_shapes_follow_layout_contract():
    m = W.TINY
    w = W.make_weights(m, 1)
    assert w.wqkv[0].shape == ((4 + 2 * 2) * 64, 256) and w.wo[0].shape == (256, 256)
    assert w.wgu[1].shape == (2048, 256) and w.wd[1].shape == (256, 1024) and w.embed.shape == (32000, 256)
    assert torch.all(w.g_attn[0] == 1) and w.w_head.dtype == torch.float32
    assert abs(w.wgu[0].float().std().item() - 0.02) < 1e-3
    j = W.make_weights(m, 1, gain_jitter=0.1)
    assert 0.05 < (j.g_mlp[1] - 1).std().item() < 0.15
    assert torch.equal(j.g_mlp[1], j.g_mlp[1].bfloat16().float())         # bf16-representable
