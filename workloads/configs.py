"""The five synthetic workloads (model shapes + batch recipes).

These stand in for the paper's math-reasoning traces (Section 5.1: LLaMA-3 /
Qwen2.5-Math families, a 1.5B router, steps delimited by a separator): only the
shapes and the length mix are reproduced; weights are random-init and token ids
are uniform.  This module holds descriptions only; `generate.py` turns them into
arrays.  Neither file contains any of the method's arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0
    kv_block: int = 16
    has_router_head: bool = True

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def params_per_layer(self) -> int:
        d, f = self.d_model, self.d_ffn
        return self.qkv_rows * d + d * self.n_q_heads * self.head_dim + 3 * d * f


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelShape
    batch: int
    prefix: Tuple[int, int]            # inclusive range; lo == hi means uniform length
    step: Tuple[str, int, int]         # ("fixed", s, s) | ("uniform", lo, hi) | ("alternate", a, b)
    tables: str                        # "identity" (contiguous KV) | "shuffled"
    kv_source: str                     # "prefill" (real prefix KV) | "synthetic"
    kv_sigma: float                    # std of synthetic prefix K/V entries
    tau: Tuple[str, float]             # ("const", v) | ("normal", std)
    seed: int
    spare_block_frac: float = 0.10     # never-referenced pool blocks (must stay untouched)
    pool_mode: str = "mean"


TINY = ModelShape("tiny-router", 2, 256, 4, 2, 64, 1024, 32000)
ROUTER_1P5B = ModelShape("router-1.5B-shape", 28, 1536, 12, 2, 128, 8960, 151936)
TARGET_8B = ModelShape("target-8B-shape", 32, 4096, 32, 8, 128, 14336, 128256, has_router_head=False)

_SEED0 = 0xA5B17

C1 = Workload("C1-tiny", TINY, 4, (512, 512), ("fixed", 32, 32), "shuffled", "prefill", 0.0,
              ("const", 0.0), _SEED0 + 0)
C2 = Workload("C2-router1.5B-b16-p2048-s64", ROUTER_1P5B, 16, (2048, 2048), ("fixed", 64, 64),
              "shuffled", "synthetic", 0.8, ("const", 0.0), _SEED0 + 1)
C3 = Workload("C3-target8B-b8-p4096-s64", TARGET_8B, 8, (4096, 4096), ("fixed", 64, 64),
              "identity", "synthetic", 1.28, ("const", 0.0), _SEED0 + 2, spare_block_frac=0.0)
C4 = Workload("C4-router1.5B-ragged-b64", ROUTER_1P5B, 64, (1024, 16384), ("uniform", 16, 128),
              "shuffled", "synthetic", 0.8, ("normal", 0.5), _SEED0 + 3)
C5 = Workload("C5-target8B-decode-mix-b32", TARGET_8B, 32, (4096, 32768), ("alternate", 1, 64),
              "shuffled", "synthetic", 1.28, ("const", 0.0), _SEED0 + 4)

ALL = {"C1": C1, "C2": C2, "C3": C3, "C4": C4, "C5": C5}


def scaled(w: Workload, *, n_layers: Optional[int] = None, batch: Optional[int] = None,
           name: Optional[str] = None) -> Workload:
    """A reduced variant (fewer layers / sequences) of a workload with the same
    per-layer shapes, for cases a CPU check has to finish in seconds."""
    m = w.model if n_layers is None else replace(w.model, n_layers=n_layers)
    return replace(w, model=m, batch=w.batch if batch is None else batch,
                   name=name or f"{w.name}[L{m.n_layers},B{batch or w.batch}]")
