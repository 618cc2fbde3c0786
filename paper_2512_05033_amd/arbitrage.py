"""Algorithm 1 (Arbitrage inference) for a batch of questions, driven from the host
over the library's calls: draft steps and target steps by arb_prefill +
arb_next_token + arb_first_stop, the routing decision by arb_score_steps.

All arithmetic runs in the library's kernels; this module only sequences the calls
and keeps the token lists.  Within a step the decode loop stays on the device (a
chosen token is fed back as the next call's input without a host copy); the host
reads back one length per sequence and step, and the router's decisions.

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

    def _forward(self, role: Role, seqs: List[int], tokens: Dict[int, List[int]], device_last: Optional[torch.Tensor],
                 score: bool = False, step: Optional[Dict[int, List[int]]] = None, feed_all: bool = False):
        """Feeds every sequence the part of `tokens[b]` its cache does not hold yet (at least the last
        token, whose hidden state gives the next token; with `feed_all` exactly the missing part), or,
        with `score`, the step on top of a fully cached context.  Returns the call's outputs and the row
        of each sequence's last token."""
        prefix, new = [], []
        for b in seqs:
            have = _lcp(role.fed.get(b, []), tokens[b])
            if score:
                assert have == len(tokens[b]), "the router's cache must hold the whole context before scoring"
                prefix.append(have)
                new.append(step[b])
            else:
                have = have if feed_all else min(have, len(tokens[b]) - 1)
                assert have < len(tokens[b])
                prefix.append(have)
                new.append(tokens[b][have:])
        lens = np.array([len(t) for t in new], np.int32)
        if int((np.array(prefix) + lens).max()) > self.capacity:
            raise RuntimeError("context exceeds the block tables")
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        if device_last is not None and bool((lens == 1).all()):
            ids = device_last                                    # decode: the tokens just chosen, still on the device
        else:
            ids = np.concatenate([np.asarray(t, np.int32) for t in new])
        batch = A.DeviceBatch(np.array(prefix, np.int32), cu, self.tables[seqs], ids, self.device)
        for b, t in zip(seqs, new):
            role.fed[b] = list(tokens[b]) + (list(t) if score else [])
        last_rows = torch.from_numpy((cu[1:] - 1).astype(np.int32)).to(self.device)
        if score:
            scores, esc, _ = A.arb_score_steps(role.model, role.kv, batch, self.tau)
            return scores, esc
        hidden = A.arb_prefill(role.model, role.kv, batch, want_hidden=True)
        return hidden, last_rows

    def _generate_step(self, role: Role, seqs: List[int], ctx: Dict[int, List[int]]) -> Dict[int, List[int]]:
        """One reasoning step per sequence: tokens until the first separator / eos, at most S."""
        n = len(seqs)
        out = torch.empty(n, self.S, dtype=torch.int32, device=self.device)
        cur = {b: list(ctx[b]) for b in seqs}
        last = None
        for i in range(self.S):
            hidden, rows = self._forward(role, seqs, cur, last)
            u = None
            if self.temperature > 0:
                u = torch.from_numpy(self.rng.random(n).astype(np.float32)).to(self.device)
            last, _ = A.arb_next_token(hidden, rows, role.w_lm, self.temperature, u)
            out[:, i] = last
            for b in seqs:                                        # placeholder ids: the host learns them after the step
                cur[b].append(-1 - i)
        length, _ = A.arb_first_stop(out, self.sep, self.eos)
        length, toks = length.cpu().numpy(), out.cpu().numpy()
        steps = {b: [int(t) for t in toks[j, :length[j]]] for j, b in enumerate(seqs)}
        for j, b in enumerate(seqs):
            # what the cache really holds: the context and the generated tokens that were fed back
            role.fed[b] = list(ctx[b]) + [int(t) for t in toks[j, :self.S - 1]]
            if self.trace is not None:
                self.trace.append(("step", role.name, b, list(ctx[b]), steps[b]))
        return steps

    # ------------------------------------------------------------------- Algorithm 1

    def run(self, questions: List[List[int]], max_steps: int):
        ctx = {b: list(q) for b, q in enumerate(questions)}
        log: Dict[int, list] = {b: [] for b in ctx}
        for _ in range(max_steps):
            active = [b for b in ctx if ctx[b][-1] != self.eos and len(ctx[b]) + self.S <= self.capacity]
            if not active:
                break
            z_d = self._generate_step(self.draft, active, ctx)
            behind = [b for b in active if _lcp(self.router.fed.get(b, []), ctx[b]) < len(ctx[b])]
            if behind:                                            # the router has not seen the last chosen step (or the question)
                self._forward(self.router, behind, ctx, None, feed_all=True)
            scores, esc = self._forward(self.router, active, ctx, None, score=True, step=z_d)
            scores, esc = scores.cpu().numpy(), esc.cpu().numpy()
            up = [b for b, e in zip(active, esc) if e]
            z_t = self._generate_step(self.target, up, ctx) if up else {}
            for j, b in enumerate(active):
                if self.trace is not None:
                    self.trace.append(("route", b, list(ctx[b]), z_d[b], float(scores[j]), bool(esc[j])))
                log[b].append((float(scores[j]), bool(esc[j])))
                ctx[b] = ctx[b] + (z_t[b] if esc[j] else z_d[b])
        return [ctx[b] for b in sorted(ctx)], log
