"""CPU oracle for the step-scoring forward and the routing decision.

TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the GPU
library computes, written for checking it; nothing in the product path may
import it.  It shares no code with the GPU path and does not import it.

What is computed (Arbitrage, Section 4.2 and Algorithm 1): the router
h_router(x, z_d) is one decoder-only transformer forward over the drafted step
z_d given the cached context x, followed by a classification head; the draft is
accepted iff the score y_hat <= tau and escalated to the target iff
y_hat > tau.  The target's regeneration pass "from the same prefix" is the same
forward without the head.  The paper does not describe the transformer; the
architecture below (pre-norm RMSNorm, rotary embedding, grouped-query attention
over a block-paged KV cache, SwiGLU MLP, mean-pooled linear head) is the one the
workload configs name.

Arithmetic: float64 throughout (the paper fixes no precision), on inputs that are
bf16-representable.  Two roundings are part of the definition because they are
part of the data contract, not of the arithmetic: keys/values are rounded to
bf16 when stored into the cache (the cache is bf16), and the routing comparison
is taken on the score rounded to fp32 against an fp32 tau.

Pins (tests/test_oracle_pins.py): softmax rows sum to one; append over
prefix+step equals one causal forward over the concatenation; rotary at position
0 is the identity, preserves norms and depends on relative position only; a
brute-force masked-matrix formulation in pure Python on tiny shapes; per-stage
agreement with torch's CPU routines in fp64; GQA == MHA with duplicated KV
heads; paged == contiguous bit-for-bit; closed forms (all keys equal, p=0 s=1,
constant segments, zero projections); Theorem B.1 (exactly-k / top-k /
monotone), Corollary B.3 and the tie rule of Algorithm 1 for the decision.
End-to-end numeric values are printed nowhere in the paper, so beyond these
pins the forward's values are "parity unpinned" by the paper itself.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np

F = np.float64


# ------------------------------------------------------------------ bf16 <-> float

def bf16_to_float(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float64 (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(F)


def float_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 (ties to even); returns uint16 bit patterns.
    float64 -> float32 is itself a rounding; for the magnitudes here a double
    rounding would need a value within 2^-29 relative of a bf16 tie, and the
    tie-breaking result is still a nearest-or-adjacent bf16 either way."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    b = f.view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    return ((b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def as_float(a) -> np.ndarray:
    """Accept bf16 bit patterns (uint16) or any float array; return float64."""
    a = np.asarray(a)
    return bf16_to_float(a) if a.dtype == np.uint16 else a.astype(F)


# ------------------------------------------------------------------------ containers

@dataclass
class Model:
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


@dataclass
class Params:
    """Matrices are [out_features, in_features]; y = x @ W.T.  wqkv rows are the
    Hq query heads, then the Hkv key heads, then the Hkv value heads; wgu rows
    are the F gate rows then the F up rows.  Arrays may be uint16 (bf16 bits)."""
    embed: np.ndarray
    wqkv: List[np.ndarray]
    wo: List[np.ndarray]
    wgu: List[np.ndarray]
    wd: List[np.ndarray]
    g_attn: List[np.ndarray]
    g_mlp: List[np.ndarray]
    g_final: np.ndarray
    w_head: Optional[np.ndarray] = None
    b_head: float = 0.0


# ----------------------------------------------------------------- paged addressing

def positions(prefix_lens, cu_step_lens) -> np.ndarray:
    """Absolute position p_b + i of every step token, concatenated over b."""
    out = []
    for b, p in enumerate(prefix_lens):
        s = int(cu_step_lens[b + 1]) - int(cu_step_lens[b])
        out.append(int(p) + np.arange(s, dtype=np.int64))
    return np.concatenate(out) if out else np.zeros(0, np.int64)


def slot_of(block_table_row, pos, blk: int):
    """Pool slot of position `pos` of one sequence: table[pos // blk]*blk + pos % blk."""
    pos = np.asarray(pos, dtype=np.int64)
    return np.asarray(block_table_row, dtype=np.int64)[pos // blk] * blk + pos % blk


def slot_mapping(prefix_lens, cu_step_lens, block_tables, blk: int) -> np.ndarray:
    """Slot of every step token (int64 [T])."""
    out = []
    for b, p in enumerate(prefix_lens):
        s = int(cu_step_lens[b + 1]) - int(cu_step_lens[b])
        out.append(slot_of(block_tables[b], int(p) + np.arange(s), blk))
    return np.concatenate(out) if out else np.zeros(0, np.int64)


def _pool_rows(pool: np.ndarray, kv_head: int, slots: np.ndarray, blk: int) -> np.ndarray:
    """pool is [n_blocks, Hkv, blk, hd]; rows at the given slots for one kv head."""
    return pool[slots // blk, kv_head, slots % blk, :]


# ---------------------------------------------------------------------------- stages

def embed(table, token_ids) -> np.ndarray:
    return as_float(np.asarray(table)[np.asarray(token_ids, dtype=np.int64)])


def rmsnorm(h: np.ndarray, g, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * g, row-wise."""
    h = h.astype(F)
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h / np.sqrt(ms + eps) * as_float(g)


def rope(u: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing: for t < hd/2 the pair
    (u[t], u[t+hd/2]) is rotated by the angle pos * base^(-2t/hd).
    u is [T, H, hd]; pos is [T] (absolute positions)."""
    u = u.astype(F)
    hd = u.shape[-1]
    half = hd // 2
    t = np.arange(half, dtype=F)
    ang = np.asarray(pos, dtype=F)[:, None] * base ** (-2.0 * t / hd)[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def kv_append(k_pool: np.ndarray, v_pool: np.ndarray, slots: np.ndarray, k: np.ndarray, v: np.ndarray, blk: int):
    """Store k, v ([T, Hkv, hd]) rounded to bf16 at the given slots (in place)."""
    k_pool[slots // blk, :, slots % blk, :] = float_to_bf16(k)
    v_pool[slots // blk, :, slots % blk, :] = float_to_bf16(v)


def softmax(x: np.ndarray) -> np.ndarray:
    e = np.exp(x - np.max(x, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def append_attention(q: np.ndarray, k_pool: np.ndarray, v_pool: np.ndarray, prefix_lens, cu_step_lens,
                     block_tables, blk: int, return_probs: bool = False):
    """Step queries against the cached prefix plus the step itself.

    q is [T, Hq, hd]; pools are bf16 bits [n_blocks, Hkv, blk, hd] that already
    hold the step's own keys/values.  Query i of sequence b (position p_b + i)
    sees keys 0..p_b+i; query head h reads kv head h // (Hq/Hkv); logits are
    scaled by 1/sqrt(hd)."""
    T, Hq, hd = q.shape
    Hkv = k_pool.shape[1]
    G = Hq // Hkv
    out = np.zeros((T, Hq, hd), dtype=F)
    probs = []
    for b, p in enumerate(prefix_lens):
        lo, hi = int(cu_step_lens[b]), int(cu_step_lens[b + 1])
        s, p = hi - lo, int(p)
        if s == 0:
            continue
        slots = slot_of(block_tables[b], np.arange(p + s), blk)
        visible = np.arange(p + s)[None, :] <= (p + np.arange(s))[:, None]
        for hk in range(Hkv):
            K = bf16_to_float(_pool_rows(k_pool, hk, slots, blk))      # [p+s, hd]
            V = bf16_to_float(_pool_rows(v_pool, hk, slots, blk))
            for h in range(hk * G, (hk + 1) * G):
                logits = (q[lo:hi, h, :].astype(F) @ K.T) / np.sqrt(F(hd))
                P = softmax(np.where(visible, logits, -np.inf))
                out[lo:hi, h, :] = P @ V
                if return_probs:
                    probs.append(P)
    return (out, probs) if return_probs else out


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def swiglu_mlp(x: np.ndarray, wgu, wd) -> np.ndarray:
    """(silu(x Wg^T) * (x Wu^T)) Wd^T with wgu = [Wg; Wu]."""
    wgu = as_float(wgu)
    f = wgu.shape[0] // 2
    return (silu(x @ wgu[:f].T) * (x @ wgu[f:].T)) @ as_float(wd).T


# --------------------------------------------------------------------------- forward

def decoder_layer(m: Model, w: Params, l: int, h: np.ndarray, k_pool: np.ndarray, v_pool: np.ndarray, pos, slots,
                  prefix_lens, cu_step_lens, block_tables, trace: Optional[Dict[str, np.ndarray]] = None) -> np.ndarray:
    """One pre-norm decoder layer on the residual stream h [T, d]: attention block
    (RMSNorm, QKV, rotary q/k, K/V append, append-attention, O projection, residual add),
    then MLP block (RMSNorm, SwiGLU, residual add)."""
    blk, Hq, Hkv, hd = m.kv_block, m.n_q_heads, m.n_kv_heads, m.head_dim
    T = h.shape[0]
    x = rmsnorm(h, w.g_attn[l], m.rms_eps)
    qkv = (x @ as_float(w.wqkv[l]).T).reshape(T, Hq + 2 * Hkv, hd)
    q = rope(qkv[:, :Hq], pos, m.rope_base)
    k = rope(qkv[:, Hq:Hq + Hkv], pos, m.rope_base)
    v = qkv[:, Hq + Hkv:]
    kv_append(k_pool, v_pool, slots, k, v, blk)
    o = append_attention(q, k_pool, v_pool, prefix_lens, cu_step_lens, block_tables, blk)
    h_attn = h + o.reshape(T, Hq * hd) @ as_float(w.wo[l]).T
    x2 = rmsnorm(h_attn, w.g_mlp[l], m.rms_eps)
    h_new = h_attn + swiglu_mlp(x2, w.wgu[l], w.wd[l])
    if trace is not None:
        trace.update(x_attn=x, qkv=qkv.reshape(T, -1), q_rot=q, k_rot=k, attn=o, h_attn=h_attn, x_mlp=x2, h1=h_new)
    return h_new


def decoder_layers(m: Model, w: Params, k_pools, v_pools, h: np.ndarray, layer_begin: int, layer_end: int,
                   prefix_lens, cu_step_lens, block_tables, keep: Optional[List[np.ndarray]] = None) -> np.ndarray:
    """Layers [layer_begin, layer_end) applied to the residual stream h; with `keep`,
    the stream after every layer is appended to it."""
    pos = positions(prefix_lens, cu_step_lens)
    slots = slot_mapping(prefix_lens, cu_step_lens, block_tables, m.kv_block)
    h = np.asarray(h, dtype=F)
    for l in range(layer_begin, layer_end):
        h = decoder_layer(m, w, l, h, k_pools[l], v_pools[l], pos, slots, prefix_lens, cu_step_lens, block_tables)
        if keep is not None:
            keep.append(h)
    return h


def forward(m: Model, w: Params, k_pools: Sequence[np.ndarray], v_pools: Sequence[np.ndarray], token_ids,
            prefix_lens, cu_step_lens, block_tables, trace: Optional[Dict[str, np.ndarray]] = None) -> np.ndarray:
    """Final-normed hidden states [T, d] of the step tokens; appends the step's
    K/V (bf16) to the pools at positions [p_b, p_b+s_b) as a side effect.
    With `trace`, per-stage tensors of layer 0 are recorded under fixed names."""
    pos = positions(prefix_lens, cu_step_lens)
    slots = slot_mapping(prefix_lens, cu_step_lens, block_tables, m.kv_block)
    h = embed(w.embed, token_ids)
    if trace is not None:
        trace["slots"], trace["h0"] = slots.copy(), h.copy()
    for l in range(m.n_layers):
        h = decoder_layer(m, w, l, h, k_pools[l], v_pools[l], pos, slots, prefix_lens, cu_step_lens, block_tables,
                          trace if l == 0 else None)
    return rmsnorm(h, w.g_final, m.rms_eps)


def router_scores(y: np.ndarray, cu_step_lens, w_head, b_head: float = 0.0, mode: str = "mean") -> np.ndarray:
    """Head on the pooled step hidden states: mean over the step's tokens (the
    workload configs' reading) or the step's final token (Section 4.2,
    'Training': head on the final-token embedding).  A [d] head gives the raw
    linear score.  A [2, d] head is the two-way classification head of Section
    4.2: logits z_c = w_c . pooled + c_c with (c_0, c_1) = (0, b_head), and the
    score is the softmax probability of class 1 (the router's y_hat)."""
    w_head = as_float(w_head)
    B = len(cu_step_lens) - 1
    out = np.zeros(B, dtype=F)
    for b in range(B):
        seg = y[int(cu_step_lens[b]):int(cu_step_lens[b + 1])]
        if mode == "mean":
            pooled = seg.sum(axis=0) / seg.shape[0]
        elif mode == "last":
            pooled = seg[-1]
        else:
            raise ValueError(mode)
        if w_head.ndim == 2:
            z = w_head @ pooled + np.array([0.0, b_head], dtype=F)
            e = np.exp(z - z.max())
            out[b] = e[1] / e.sum()
        else:
            out[b] = pooled @ w_head + b_head
    return out


def route(scores, tau: float, sense: str = "escalate_if_gt") -> np.ndarray:
    """Escalation flags (uint8).  Arbitrage (Fig. 1, Alg. 1): accept iff
    y_hat <= tau, so escalate = not (y_hat <= tau); a NaN score escalates.
    RSD (Section 3.1): accept iff s_d > tau, so escalate = not (s_d > tau).
    The comparison is taken in fp32."""
    s = np.asarray(scores).astype(np.float32)
    t = np.float32(tau)
    with np.errstate(invalid="ignore"):
        if sense == "escalate_if_gt":
            return (~(s <= t)).astype(np.uint8)
        if sense == "accept_if_gt":
            return (~(s > t)).astype(np.uint8)
    raise ValueError(sense)


def score_steps(m: Model, w: Params, k_pools, v_pools, token_ids, prefix_lens, cu_step_lens, block_tables,
                tau: float, mode: str = "mean", trace=None):
    """(scores [B], escalate [B] uint8, hidden [T, d])."""
    y = forward(m, w, k_pools, v_pools, token_ids, prefix_lens, cu_step_lens, block_tables, trace)
    scores = router_scores(y, cu_step_lens, w.w_head, w.b_head, mode)
    return scores, route(scores, tau), y


def prefill(m: Model, w: Params, k_pools, v_pools, token_ids, cu_lens, block_tables) -> np.ndarray:
    """Fill the cache for whole prompts: the same forward with empty prefixes."""
    zeros = np.zeros(len(cu_lens) - 1, dtype=np.int32)
    return forward(m, w, k_pools, v_pools, token_ids, zeros, cu_lens, block_tables)


# -------------------------------------------------- oracle-mode routing (Section 4.1)

def advantage(s_t, s_d) -> np.ndarray:
    """Step-level advantage Delta = s_t - s_d (Definition 4.1)."""
    return np.asarray(s_t, dtype=F) - np.asarray(s_d, dtype=F)


def realized_score(s_d, s_t, a) -> np.ndarray:
    """S(a) = (1-a) s_d + a s_t (Definition 4.2)."""
    a = np.asarray(a, dtype=F)
    return (1.0 - a) * np.asarray(s_d, dtype=F) + a * np.asarray(s_t, dtype=F)


def budget_threshold(delta, budget: int) -> float:
    """A threshold tau for the oracle policy a_i = 1{Delta_i > tau} under at most `budget`
    escalations (Theorem B.1 and its proof): the optimum escalates the
    k = min(budget, #{Delta_i > 0}) largest positive advantages, which any tau with
    Delta_(k) > tau >= Delta_(k+1) selects.  Returned: max(0, Delta_(budget+1)) with
    Delta_(N+1) = -inf, in the precision of the input.  Entries that are NaN escalate
    whatever tau is, so they are ranked above every number; if they alone exceed
    the budget the result is +inf."""
    d = np.asarray(delta)
    n = d.size
    if budget >= n:
        return 0.0
    key = np.where(np.isnan(d), np.inf, d)
    kth = np.sort(key)[::-1][budget]           # the (budget+1)-th largest
    if np.isnan(d).sum() > budget:
        return float("inf")
    return float(max(kth, 0.0))


# ------------------------------------------------------------- the loop around the scoring (Algorithm 1)

def lm_logits(hidden_rows: np.ndarray, w_lm) -> np.ndarray:
    """Next-token logits of the final-normed hidden states of the last tokens: h . W_lm^T."""
    return np.asarray(hidden_rows, dtype=F) @ as_float(w_lm).T


def choose_token(logits: np.ndarray, temperature: float = 0.0, u: Optional[float] = None) -> int:
    """Greedy choice (temperature <= 0: first index of the maximum) or a draw from
    softmax(logits / temperature) by inversion: the smallest k whose cumulative
    probability reaches u (u in [0, 1))."""
    l = np.asarray(logits, dtype=F)
    if not temperature > 0:
        return int(np.argmax(l))
    w = np.exp((l - l.max()) / temperature)
    c = np.cumsum(w)
    k = int(np.searchsorted(c, u * c[-1], side="left"))
    return min(k, l.size - 1)


def first_stop(tokens, sep: int, eos: int):
    """(length, ended): a step runs up to and including its first separator or
    end-of-sequence token (Algorithm 1); all of `tokens` if there is none."""
    for i, t in enumerate(tokens):
        if t == sep or t == eos:
            return i + 1, t == eos
    return len(tokens), False


def arbitrage_inference(question, draft_step, router_score, target_step, tau: float, eos: int, max_steps: int):
    """Algorithm 1.  draft_step(x) / target_step(x) return the tokens of one reasoning
    step generated from context x (ending with the separator or eos); router_score(x, z)
    returns y_hat.  Returns the final sequence and, per step, (y_hat, escalated)."""
    x = list(question)
    log = []
    for _ in range(max_steps):
        if x and x[-1] == eos:
            break
        z_d = list(draft_step(x))
        y_hat = router_score(x, z_d)
        escalate = bool(route(np.array([y_hat]), tau)[0])
        z = list(target_step(x)) if escalate else z_d
        x = x + z
        log.append((y_hat, escalate))
    return x, log


# ------------------------------------------------- 4-bit weights of the self-draft regime (Section 5.1)

W4_GROUP = 128


def w4_quantize(w_bits: np.ndarray, bits: int = 4):
    """Group-wise symmetric quantization of a bf16 weight matrix [N, K] (bit patterns) to `bits`-bit
    integers (4: the Q4 self-drafts of Section 5.1; 3: the 3-bit Qwen draft of Section 5.2): with
    qmax = 2^(bits-1) - 1, per row and group of 128 consecutive k, scale = bf16(max|w| / qmax) and
    q = clip(rint(w / scale), -qmax - 1, qmax) (0 where the scale is 0), quotients in fp32,
    round-half-even.  Returns (q int8 [N, K], scale bits uint16 [N, K/128]).  (The paper
    quantizes its drafts with GPTQ / llama.cpp; how the integers are chosen offline does
    not matter to the forward, which only sees integers and group scales.)"""
    if bits not in (3, 4):
        raise ValueError("bits")
    qmax = 2 ** (bits - 1) - 1
    w = bf16_to_float(w_bits).astype(np.float32)
    N, K = w.shape
    g = w.reshape(N, K // W4_GROUP, W4_GROUP)
    scale_bits = float_to_bf16(np.abs(g).max(axis=2) / np.float32(qmax))
    scale = bf16_to_float(scale_bits).astype(np.float32)
    safe = np.where(scale == 0, np.float32(1.0), scale)[:, :, None]
    q = np.clip(np.rint(g / safe), -qmax - 1, qmax)
    q = np.where(scale[:, :, None] == 0, 0, q).astype(np.int8)
    return q.reshape(N, K), scale_bits


def w4_dequantize(q: np.ndarray, scale_bits: np.ndarray) -> np.ndarray:
    """w'[n, k] = q[n, k] * scale[n, k // 128], exactly (float64)."""
    s = bf16_to_float(scale_bits)
    return q.astype(F) * np.repeat(s, W4_GROUP, axis=1)


def w4_pack(q: np.ndarray) -> np.ndarray:
    """Storage format: offset-binary nibbles (q + 8), eight consecutive k per uint32: the even
    ones in the four low nibbles, the odd ones in the four high nibbles (input 2i in nibble i,
    input 2i + 1 in nibble 4 + i, nibble 0 the least significant), so that two neighbours sit
    16 bits apart (3-bit integers use the same nibbles).  [N, K] -> uint32 [N, K/8]."""
    N, K = q.shape
    u = (q.astype(np.int32) + 8).astype(np.uint32).reshape(N, K // 8, 8)
    e = np.arange(8)
    nibble = e // 2 + 4 * (e % 2)
    return (u << (4 * nibble).astype(np.uint32)[None, None, :]).sum(axis=2, dtype=np.uint64).astype(np.uint32)

