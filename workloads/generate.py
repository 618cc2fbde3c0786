"""Seeded synthetic inputs, identical on any device.

Every large tensor (weights, token ids, synthetic prefix K/V) is a pure function
of (seed, stream name, flat element index): a 64-bit integer hash of the index
selects one of 65536 standard-normal quantiles, which is scaled and rounded to
bf16.  Integer torch ops are bit-exact on CPU and GPU and the only floating-point
operation is one IEEE fp32 multiply, so a GPU can fill an 80 GB KV pool in place
while a CPU check materialises just the blocks it needs and sees the same bits.

The hash is the splitmix64 output function (Steele, Lea & Flood 2014).  Nothing
here belongs to the method under test: no norm, rotation, attention, pooling or
comparison.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import scipy.special
import torch

from .configs import ModelShape, Workload

_CHUNK = 1 << 25          # elements hashed per pass (bounds int64 temporaries to ~1 GB)


def _s64(c: int) -> int:
    """Two's-complement int64 value of an unsigned 64-bit constant."""
    c &= (1 << 64) - 1
    return c - (1 << 64) if c >= (1 << 63) else c


_GOLDEN, _M1, _M2 = _s64(0x9E3779B97F4A7C15), _s64(0xBF58476D1CE4E5B9), _s64(0x94D049BB133111EB)


def stream_key(seed: int, name: str) -> int:
    digest = hashlib.blake2b(f"{seed}/{name}".encode(), digest_size=8).digest()
    return _s64(int.from_bytes(digest, "little"))


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    return (x >> k) & ((1 << (64 - k)) - 1)


def hash64(idx: torch.Tensor, key: int) -> torch.Tensor:
    """splitmix64 finaliser of (idx + key); int64 in, int64 out (wrapping)."""
    z = idx + key + _GOLDEN
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


_quantiles: Dict[str, torch.Tensor] = {}


def _quantile_table(device) -> torch.Tensor:
    dev = str(device)
    if dev not in _quantiles:
        k = np.arange(65536, dtype=np.float64)
        tab = scipy.special.ndtri((k + 0.5) / 65536.0).astype(np.float32)
        _quantiles[dev] = torch.from_numpy(tab).to(device)
    return _quantiles[dev]


def _to_bf16_bits(x: torch.Tensor) -> torch.Tensor:
    """fp32 -> nearest-even bf16, as int16 bit patterns (inputs are finite)."""
    b = x.view(torch.int32)
    b = b + (((b >> 16) & 1) + 0x7FFF)
    return (b >> 16).to(torch.int16)


def normal_bf16_at(seed: int, name: str, flat_idx: torch.Tensor, sigma: float) -> torch.Tensor:
    """bf16 N(0, sigma^2) draws at the given flat indices (int64 tensor)."""
    dev = flat_idx.device
    h = hash64(flat_idx, stream_key(seed, name))
    z = _quantile_table(dev)[h & 0xFFFF]
    v = z * torch.tensor(sigma, dtype=torch.float32, device=dev)
    return _to_bf16_bits(v).view(torch.bfloat16)


def normal_bf16(seed: int, name: str, shape: Sequence[int], sigma: float, device="cpu",
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
    n = int(np.prod(shape))
    if out is None:
        out = torch.empty(n, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=flat.device)
        flat[lo:hi] = normal_bf16_at(seed, name, idx, sigma)
    return flat.view(*shape)


def uniform_ints(seed: int, name: str, n: int, hi: int, device="cpu") -> torch.Tensor:
    """int32 draws in [0, hi)."""
    idx = torch.arange(n, dtype=torch.int64, device=device)
    h = _lsr(hash64(idx, stream_key(seed, name)), 1)       # non-negative
    return (h % hi).to(torch.int32)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """A bf16 tensor as a host uint16 array of its bit patterns."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


# --------------------------------------------------------------------------- weights

@dataclass
class Weights:
    """All matrices are [out_features, in_features] row-major bf16 (y = x W^T).
    wqkv rows: Hq query heads, then Hkv key heads, then Hkv value heads.
    wgu rows: F gate rows, then F up rows.  Gains and head are fp32."""
    embed: torch.Tensor
    wqkv: List[torch.Tensor]
    wo: List[torch.Tensor]
    wgu: List[torch.Tensor]
    wd: List[torch.Tensor]
    g_attn: List[torch.Tensor]
    g_mlp: List[torch.Tensor]
    g_final: torch.Tensor
    w_head: torch.Tensor
    b_head: float = 0.0


def _gain(seed: int, name: str, d: int, jitter: float, device) -> torch.Tensor:
    g = torch.ones(d, dtype=torch.float32, device=device)
    if jitter > 0.0:
        g = (g + normal_bf16(seed, name, (d,), jitter, device).float()).bfloat16().float()
    return g


def make_weights(m: ModelShape, seed: int, device="cpu", sigma: float = 0.02,
                 gain_jitter: float = 0.0, b_head: float = 0.0, two_class_head: bool = False) -> Weights:
    """Matrices, embedding and head ~ N(0, sigma^2) rounded to bf16; RMSNorm gains
    are 1 (plus an optional bf16-representable jitter, used by tests so that a
    dropped gain is visible).  two_class_head: the head is a [2, d] matrix (one row
    per class) instead of a [d] vector; b_head then stands for the bias difference."""
    d, f, hq = m.d_model, m.d_ffn, m.n_q_heads * m.head_dim
    mk = lambda name, shape: normal_bf16(seed, name, shape, sigma, device)
    return Weights(
        embed=mk("embed", (m.vocab, d)),
        wqkv=[mk(f"L{l}.wqkv", (m.qkv_rows, d)) for l in range(m.n_layers)],
        wo=[mk(f"L{l}.wo", (d, hq)) for l in range(m.n_layers)],
        wgu=[mk(f"L{l}.wgu", (2 * f, d)) for l in range(m.n_layers)],
        wd=[mk(f"L{l}.wd", (d, f)) for l in range(m.n_layers)],
        g_attn=[_gain(seed, f"L{l}.g_attn", d, gain_jitter, device) for l in range(m.n_layers)],
        g_mlp=[_gain(seed, f"L{l}.g_mlp", d, gain_jitter, device) for l in range(m.n_layers)],
        g_final=_gain(seed, "g_final", d, gain_jitter, device),
        w_head=normal_bf16(seed, "w_head", (2, d) if two_class_head else (d,), sigma, device).float(),
        b_head=b_head,
    )


# ----------------------------------------------------------------------------- batch

@dataclass
class Batch:
    """Host-side description of one call: B sequences, each a cached prefix of
    prefix_lens[b] tokens plus a step of cu_step_lens[b+1]-cu_step_lens[b] tokens."""
    prefix_lens: np.ndarray      # int32 [B]
    cu_step_lens: np.ndarray     # int32 [B+1]
    block_tables: np.ndarray     # int32 [B, max_blocks_per_seq]
    token_ids: np.ndarray        # int32 [T]
    n_blocks: int                # pool size in blocks
    kv_block: int
    tau: float
    spare_blocks: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))

    @property
    def batch(self) -> int:
        return len(self.prefix_lens)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_step_lens[-1])

    @property
    def step_lens(self) -> np.ndarray:
        return np.diff(self.cu_step_lens)

    def select(self, rows: Sequence[int]) -> "Batch":
        """The sub-batch made of the given sequences, against the same pool."""
        rows = list(rows)
        s = self.step_lens[rows]
        cu = np.concatenate([[0], np.cumsum(s)]).astype(np.int32)
        tok = np.concatenate([self.token_ids[self.cu_step_lens[b]:self.cu_step_lens[b + 1]] for b in rows])
        return Batch(self.prefix_lens[rows].copy(), cu, self.block_tables[rows].copy(), tok.astype(np.int32),
                     self.n_blocks, self.kv_block, self.tau, self.spare_blocks)


def make_batch(w: Workload, *, prefix_lens: Optional[Sequence[int]] = None,
               step_lens: Optional[Sequence[int]] = None) -> Batch:
    rng = np.random.default_rng(w.seed)
    B, blk = w.batch, w.model.kv_block
    if prefix_lens is None:
        lo, hi = w.prefix
        prefix_lens = rng.integers(lo, hi + 1, size=B) if hi > lo else np.full(B, lo)
    if step_lens is None:
        kind, a, b = w.step
        if kind == "fixed":
            step_lens = np.full(B, a)
        elif kind == "uniform":
            step_lens = rng.integers(a, b + 1, size=B)
        elif kind == "alternate":       # even sequence index: a tokens; odd: b tokens
            step_lens = np.where(np.arange(B) % 2 == 0, a, b)
        else:
            raise ValueError(kind)
    p = np.asarray(prefix_lens, dtype=np.int32)
    s = np.asarray(step_lens, dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum(s)]).astype(np.int32)
    need = (p + s + blk - 1) // blk
    used = int(need.sum())
    n_blocks = used + int(np.ceil(used * w.spare_block_frac))
    if w.tables == "shuffled":
        ids = rng.permutation(n_blocks).astype(np.int32)
    elif w.tables == "identity":
        ids = np.arange(n_blocks, dtype=np.int32)
    else:
        raise ValueError(w.tables)
    spare = np.sort(ids[used:])
    max_blocks = int(need.max())
    # table entries past a sequence's need point at a spare block (or block 0): a
    # stray access lands in memory the checks watch instead of out of bounds
    filler = int(spare[0]) if len(spare) else 0
    tables = np.full((B, max_blocks), filler, dtype=np.int32)
    at = 0
    for b in range(B):
        tables[b, :need[b]] = ids[at:at + need[b]]
        at += need[b]
    tok = uniform_ints(w.seed, "step_token_ids", int(cu[-1]), w.model.vocab).numpy()
    kind, v = w.tau
    tau = float(v) if kind == "const" else float(np.float32(rng.normal(0.0, v)))
    return Batch(p, cu, tables, tok, n_blocks, blk, tau, spare)


def prompt_token_ids(w: Workload, batch: Batch) -> np.ndarray:
    """Ids of the prefix tokens (concatenated over sequences), for workloads whose
    prefix K/V comes from a real prefill."""
    return uniform_ints(w.seed, "prefix_token_ids", int(batch.prefix_lens.sum()), w.model.vocab).numpy()


# -------------------------------------------------------------------------- KV pools

def kv_pool_shape(m: ModelShape, n_blocks: int):
    return (n_blocks, m.n_kv_heads, m.kv_block, m.head_dim)


def _kv_sigma(w: Workload) -> float:
    return w.kv_sigma if w.kv_source == "synthetic" else 1.0   # prefill case: filler to be overwritten


def make_kv_pools(w: Workload, batch: Batch, device="cpu"):
    """Per-layer K and V pools, bf16 [n_blocks, Hkv, kv_block, head_dim], every
    element filled from its stream (for a 'prefill' workload this is filler that a
    prefill must overwrite wherever it is later read)."""
    shape = kv_pool_shape(w.model, batch.n_blocks)
    ks = [normal_bf16(w.seed, f"L{l}.kpool", shape, _kv_sigma(w), device) for l in range(w.model.n_layers)]
    vs = [normal_bf16(w.seed, f"L{l}.vpool", shape, _kv_sigma(w), device) for l in range(w.model.n_layers)]
    return ks, vs


def kv_pool_blocks(w: Workload, layer: int, which: str, block_ids: Sequence[int], device="cpu") -> torch.Tensor:
    """The same values as make_kv_pools()[which][layer][block_ids], without
    building the pool: bf16 [len(block_ids), Hkv, kv_block, head_dim]."""
    m = w.model
    per_block = m.n_kv_heads * m.kv_block * m.head_dim
    ids = torch.as_tensor(np.asarray(block_ids), dtype=torch.int64, device=device)
    idx = (ids[:, None] * per_block + torch.arange(per_block, dtype=torch.int64, device=device)[None, :]).reshape(-1)
    vals = normal_bf16_at(w.seed, f"L{layer}.{which}pool", idx, _kv_sigma(w))
    return vals.view(len(ids), m.n_kv_heads, m.kv_block, m.head_dim)
