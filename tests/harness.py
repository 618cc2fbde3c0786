"""Builds device-resident inputs of a seeded workload for the tests, the smoke
check and the benchmark.  Not part of the hot path: it only allocates tensors
and wraps them for the binding."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

import workloads as W

import paper_2512_05033_amd as A


@dataclass
class Session:
    workload: W.Workload
    batch: W.Batch
    weights: W.Weights
    model: A.Model
    kv: A.KVCache
    dbatch: A.DeviceBatch
    ws: torch.Tensor


def make_model(m: W.ModelShape, weights: W.Weights, pool: int = A.ARB_POOL_MEAN,
               has_router_head: Optional[bool] = None) -> A.Model:
    return A.Model(n_layers=m.n_layers, d_model=m.d_model, n_q_heads=m.n_q_heads, n_kv_heads=m.n_kv_heads,
                   head_dim=m.head_dim, d_ffn=m.d_ffn, vocab=m.vocab, weights=weights, rms_eps=m.rms_eps,
                   rope_base=m.rope_base, kv_block=m.kv_block, pool=pool,
                   has_router_head=m.has_router_head if has_router_head is None else has_router_head)


def device_batch(batch: W.Batch, device="cuda") -> A.DeviceBatch:
    return A.DeviceBatch(batch.prefix_lens, batch.cu_step_lens, batch.block_tables, batch.token_ids, device)


def prompt_batch(w: W.Workload, batch: W.Batch, device="cuda") -> A.DeviceBatch:
    """The prefill call that produces a 'prefill' workload's prefix K/V."""
    cu = np.concatenate([[0], np.cumsum(batch.prefix_lens)]).astype(np.int32)
    return A.DeviceBatch(np.zeros(batch.batch, np.int32), cu, batch.block_tables, W.prompt_token_ids(w, batch), device)


def setup(w: W.Workload, device="cuda", *, gain_jitter: float = 0.0, sigma: float = 0.02, b_head: float = 0.0,
          pool: int = A.ARB_POOL_MEAN, batch: Optional[W.Batch] = None, two_class_head: bool = False) -> Session:
    batch = batch or W.make_batch(w)
    weights = W.make_weights(w.model, w.seed, device, sigma=sigma, gain_jitter=gain_jitter, b_head=b_head,
                             two_class_head=two_class_head)
    model = make_model(w.model, weights, pool)
    ks, vs = W.make_kv_pools(w, batch, device)
    kv = A.KVCache(ks, vs)
    db = device_batch(batch, device)
    max_tokens = max(batch.total_tokens, int(batch.prefix_lens.sum()) if w.kv_source == "prefill" else 0)
    ws = torch.empty(model.workspace_bytes(batch.batch, max_tokens, db.max_ctx), dtype=torch.uint8, device=device)
    sess = Session(w, batch, weights, model, kv, db, ws)
    if w.kv_source == "prefill":
        A.arb_prefill(model, kv, prompt_batch(w, batch, device), ws=ws)
    return sess
