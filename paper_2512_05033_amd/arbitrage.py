"""Algorithm 1 (Arbitrage inference) for a batch of questions, driven from the host
over the library's calls: draft steps and target steps by arb_prefill +
arb_next_token + arb_first_stop, the routing decision by arb_score_steps.

All arithmetic runs in the library's kernels; this module only sequences the calls
and keeps the token lists.  Within a step the decode loop keeps the tokens on the
device: a chosen token is appended to its step and fed back by arb_step_advance,
steps that reach their separator drop out of the batch, the loop ends when none is
open, and the router scores the drafted steps from the device copy
(arb_pack_steps).  The host reads back the list of open rows per token position,
the step lengths and the router's decisions, and the tokens once per step.

Lengths are stateless: a model's cache is valid for the longest common prefix of
what it has been fed and the sequence it is asked to continue, so rejecting a
draft step costs nothing but the positions being overwritten later.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as A


@dataclass
class Role:
    """One of the three models of Alg. 1 with its own KV cache.  w_lm (bf16 [vocab, d]) is needed
    by the draft and the target, not by the router."""
    name: str
    model: A.Model
    kv: A.KVCache
    w_lm: Optional[torch.Tensor] = None
    fed: Dict[int, List[int]] = field(default_factory=dict)      # per sequence: tokens whose K/V the cache holds


def _lcp(a: Sequence[int], b: Sequence[int]) -> int:
    n = 0
    for x, y in zip(a, b):
        if x != y:
            break
        n += 1
    return n


class Arbitrage:
    def __init__(self, draft: Role, target: Role, router: Role, block_tables: np.ndarray, *, tau: float, sep: int,
                 eos: int, max_step_tokens: int, temperature: float = 0.0, seed: int = 0, trace: Optional[list] = None):
        self.draft, self.target, self.router = draft, target, router
        self.tables = np.ascontiguousarray(block_tables, dtype=np.int32)
        self.tau, self.sep, self.eos, self.S = float(tau), int(sep), int(eos), int(max_step_tokens)
        self.temperature = float(temperature)
        self.rng = np.random.default_rng(seed)
        self.trace = trace
        self.device = draft.model.device
        self.capacity = self.tables.shape[1] * draft.model.cfg.kv_block

    # ------------------------------------------------------------------ model calls

    def _forward(self, role: Role, seqs: List[int], tokens: Dict[int, List[int]], feed_all: bool = False):
        """Feeds every sequence the part of `tokens[b]` its cache does not hold yet (at least the last
        token, whose hidden state gives the next token; with `feed_all` exactly the missing part).
        Returns the hidden states and the row of each sequence's last token."""
        prefix, new = [], []
        for b in seqs:
            have = _lcp(role.fed.get(b, []), tokens[b])
            have = have if feed_all else min(have, len(tokens[b]) - 1)
            assert have < len(tokens[b])
            prefix.append(have)
            new.append(tokens[b][have:])
        lens = np.array([len(t) for t in new], np.int32)
        if int((np.array(prefix) + lens).max()) > self.capacity:
            raise RuntimeError("context exceeds the block tables")
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        ids = np.concatenate([np.asarray(t, np.int32) for t in new])
        batch = A.DeviceBatch(np.array(prefix, np.int32), cu, self.tables[seqs], ids, self.device)
        for b in seqs:
            role.fed[b] = list(tokens[b])
        last_rows = torch.from_numpy((cu[1:] - 1).astype(np.int32)).to(self.device)
        hidden = A.arb_prefill(role.model, role.kv, batch, want_hidden=True)
        return hidden, last_rows

    def _generate_step(self, role: Role, seqs: List[int], ctx: Dict[int, List[int]]):
        """One reasoning step per sequence: tokens until the first separator / eos, at most S.  Returns the
        device state of the steps (tokens int32 [n, S], lengths int32 [n]) and the lengths on the host.

        The decode loop keeps every token on the device: arb_next_token's choice goes through
        arb_step_advance, which appends it to its step, closes steps that end and hands back the ids of the
        next iteration together with the rows still open; the host reads that short list (one small copy per
        token position) to size the next call, so finished steps cost no further forward work and the loop
        ends when all steps have ended."""
        n = len(seqs)
        dev = self.device
        steps = torch.zeros(n, self.S, dtype=torch.int32, device=dev)
        length = torch.zeros(n, dtype=torch.int32, device=dev)
        done = torch.zeros(n, dtype=torch.uint8, device=dev)
        open_rows = list(range(n))
        open_dev = torch.arange(n, dtype=torch.int32, device=dev)
        next_buf = torch.empty(1 + n, dtype=torch.int32, device=dev)
        next_ids = torch.empty(n, dtype=torch.int32, device=dev)
        for i in range(self.S):
            if i == 0:
                hidden, rows = self._forward(role, seqs, ctx)                # the uncached tail of the context
            else:
                # one token per open row: the one chosen last (still on the device), on top of the context and the
                # i - 1 generated tokens the cache already holds
                rows_b = [seqs[r] for r in open_rows]
                prefix = np.array([len(ctx[b]) + i - 1 for b in rows_b], np.int32)
                if int(prefix.max()) + 1 > self.capacity:
                    raise RuntimeError("context exceeds the block tables")
                cu = np.arange(len(rows_b) + 1, dtype=np.int32)
                batch = A.DeviceBatch(prefix, cu, self.tables[rows_b], next_ids[:len(rows_b)], dev)
                hidden = A.arb_prefill(role.model, role.kv, batch, want_hidden=True)
                rows = torch.arange(len(rows_b), dtype=torch.int32, device=dev)
            u = None
            if self.temperature > 0:
                u = torch.from_numpy(self.rng.random(len(open_rows)).astype(np.float32)).to(dev)
            last, _ = A.arb_next_token(hidden, rows, role.w_lm, self.temperature, u)
            A.arb_step_advance(open_dev, last, steps, length, done, self.sep, self.eos, next_buf, next_ids)
            nb = next_buf[:1 + len(open_rows)].cpu().numpy()                  # the one read-back of this token position
            open_rows = [int(r) for r in nb[1:1 + int(nb[0])]]
            if not open_rows:
                break
            open_dev = next_buf[1:1 + len(open_rows)].clone()
        return steps, length, length.cpu().numpy()

    def _read_steps(self, role: Role, seqs: List[int], ctx: Dict[int, List[int]], steps: torch.Tensor,
                    lens: np.ndarray) -> Dict[int, List[int]]:
        """The generated steps as token lists (host), with the bookkeeping of what the role's cache holds: the
        context and every generated token that was fed back, i.e. all but a step's last one."""
        toks = steps.cpu().numpy()
        out = {}
        for j, b in enumerate(seqs):
            out[b] = [int(t) for t in toks[j, :lens[j]]]
            role.fed[b] = list(ctx[b]) + out[b][:-1]
            if self.trace is not None:
                self.trace.append(("step", role.name, b, list(ctx[b]), out[b]))
        return out

    def _score(self, seqs: List[int], ctx: Dict[int, List[int]], steps: torch.Tensor, lens: np.ndarray):
        """Router scores of the drafted steps, taken from the device-resident step tokens (arb_pack_steps): the
        router's cache must hold each context."""
        for b in seqs:
            assert _lcp(self.router.fed.get(b, []), ctx[b]) == len(ctx[b]), "the router's cache must hold the whole context before scoring"
        prefix = np.array([len(ctx[b]) for b in seqs], np.int32)
        if int((prefix + lens).max()) > self.capacity:
            raise RuntimeError("context exceeds the block tables")
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        rows = torch.arange(len(seqs), dtype=torch.int32, device=self.device)
        cu_dev = torch.from_numpy(cu).to(self.device)
        ids = A.arb_pack_steps(steps, rows, cu_dev, int(cu[-1]))
        batch = A.DeviceBatch(prefix, cu, self.tables[seqs], ids, self.device)
        scores, esc, _ = A.arb_score_steps(self.router.model, self.router.kv, batch, self.tau)
        return scores, esc

    # ------------------------------------------------------------------- Algorithm 1

    def run(self, questions: List[List[int]], max_steps: int):
        ctx = {b: list(q) for b, q in enumerate(questions)}
        log: Dict[int, list] = {b: [] for b in ctx}
        for _ in range(max_steps):
            active = [b for b in ctx if ctx[b][-1] != self.eos and len(ctx[b]) + self.S <= self.capacity]
            if not active:
                break
            d_steps, _, d_lens = self._generate_step(self.draft, active, ctx)
            behind = [b for b in active if _lcp(self.router.fed.get(b, []), ctx[b]) < len(ctx[b])]
            if behind:                                            # the router has not seen the last chosen step (or the question)
                self._forward(self.router, behind, ctx, feed_all=True)
            scores, esc = self._score(active, ctx, d_steps, d_lens)
            scores, esc = scores.cpu().numpy(), esc.cpu().numpy()
            z_d = self._read_steps(self.draft, active, ctx, d_steps, d_lens)
            for b in active:
                self.router.fed[b] = list(ctx[b]) + z_d[b]
            up = [b for b, e in zip(active, esc) if e]
            z_t = {}
            if up:
                t_steps, _, t_lens = self._generate_step(self.target, up, ctx)
                z_t = self._read_steps(self.target, up, ctx, t_steps, t_lens)
            for j, b in enumerate(active):
                if self.trace is not None:
                    self.trace.append(("route", b, list(ctx[b]), z_d[b], float(scores[j]), bool(esc[j])))
                log[b].append((float(scores[j]), bool(esc[j])))
                ctx[b] = ctx[b] + (z_t[b] if esc[j] else z_d[b])
        return [ctx[b] for b in sorted(ctx)], log
