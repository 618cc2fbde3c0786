"""Pins for the CPU oracle: what the paper and the mathematics fix, checked
against formulations that do not reuse the oracle's own code."""
import math
import struct

import numpy as np
import pytest
import torch

import workloads as W
from helpers import oracle_model, oracle_params, oracle_pools
from oracle import arb_oracle as O

RNG = np.random.default_rng(20251205)


# ----------------------------------------------------------------- small fixtures

SMALL = W.ModelShape("pin-small", 2, 32, 4, 2, 8, 48, 97, kv_block=4)
SMALL_W = W.Workload("pin-small", SMALL, 3, (5, 11), ("uniform", 1, 6), "shuffled", "prefill", 0.0,
                     ("const", 0.0), 7)


def small_case(gain_jitter=0.1, sigma=0.3):
    """A ragged 3-sequence case whose prefix lengths are not block multiples.
    sigma is large so attention is far from uniform and every term matters."""
    batch = W.make_batch(SMALL_W)
    weights = W.make_weights(SMALL, SMALL_W.seed, sigma=sigma, gain_jitter=gain_jitter, b_head=0.25)
    return batch, weights


def run_prefill_then_step(batch, weights, model=SMALL, wl=SMALL_W):
    m, p = oracle_model(model), oracle_params(weights)
    kp, vp = oracle_pools(*W.make_kv_pools(wl, batch))
    prompt = W.prompt_token_ids(wl, batch)
    cu_p = np.concatenate([[0], np.cumsum(batch.prefix_lens)]).astype(np.int32)
    O.prefill(m, p, kp, vp, prompt, cu_p, batch.block_tables)
    scores, esc, y = O.score_steps(m, p, kp, vp, batch.token_ids, batch.prefix_lens, batch.cu_step_lens,
                                   batch.block_tables, batch.tau)
    return m, p, kp, vp, prompt, scores, esc, y


# ------------------------------------------------------------- bf16 conversion pins

def test_bf16_round_matches_torch_and_struct():
    x = np.concatenate([RNG.normal(0, 1, 4096), RNG.normal(0, 1e-3, 512), [0.0, -0.0, 1.0, 1.00390625, 1.01171875]])
    got = O.float_to_bf16(x)
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)
    # widening: bf16 bits are the top half of the fp32 pattern
    for bits in (0x3F80, 0xBF80, 0x4049, 0x0080, 0x7F7F):
        want = struct.unpack("<f", struct.pack("<I", bits << 16))[0]
        assert O.bf16_to_float(np.array([bits], np.uint16))[0] == want
    # ties go to even: 1 + 2^-8 is halfway between 1.0 (even) and 1 + 2^-7
    assert O.float_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 0x3F80
    assert O.float_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 0x3F82


# ------------------------------------------------------------------ paged addressing

def test_slot_mapping_brute_force():
    blk = 4
    tables = np.array([[7, 2, 9, 0], [5, 1, 3, 8]], np.int32)
    prefix, cu = np.array([6, 3], np.int32), np.array([0, 5, 9], np.int32)
    want = []
    for b in range(2):
        for i in range(cu[b + 1] - cu[b]):
            pos = prefix[b] + i
            want.append(tables[b][pos // blk] * blk + pos % blk)
    assert O.slot_mapping(prefix, cu, tables, blk).tolist() == want
    # hand-worked: seq 0 positions 6..10 -> blocks 2,2,9,9,9 -> 8+2, 8+3, 36+0, 36+1, 36+2
    assert want[:5] == [10, 11, 36, 37, 38]
    assert O.positions(prefix, cu).tolist() == [6, 7, 8, 9, 10, 3, 4, 5, 6]


# ------------------------------------------------------------------------------ RMSNorm

def test_rmsnorm_closed_forms_and_torch():
    h = RNG.normal(0, 3, (5, 64))
    y = O.rmsnorm(h, np.ones(64), 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0, atol=1e-12)          # unit rms
    assert np.allclose(O.rmsnorm(7.5 * h, np.ones(64), 0.0), y, atol=1e-12)         # scale invariance
    g = RNG.normal(1, 0.2, 64)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(h), (64,), torch.from_numpy(g), eps=1e-6).numpy()
    assert np.allclose(O.rmsnorm(h, g, 1e-6), ref, atol=1e-12)
    # eps enters under the root, added to the mean square: a zero row stays zero,
    # and a row of constant c maps to c/sqrt(c^2+eps)
    assert np.all(O.rmsnorm(np.zeros((1, 8)), np.ones(8), 1e-6) == 0.0)
    assert np.allclose(O.rmsnorm(np.full((1, 8), 1e-3), np.ones(8), 1e-6), 1e-3 / math.sqrt(2e-6))


# --------------------------------------------------------------------------------- RoPE

def test_rope_identity_norm_relative():
    u = RNG.normal(0, 1, (3, 2, 16))
    assert np.array_equal(O.rope(u, np.zeros(3), 10000.0), u)                       # position 0
    r = O.rope(u, np.array([1, 77, 4099]), 10000.0)
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(u, axis=-1), atol=1e-12)
    q, k = RNG.normal(0, 1, (1, 1, 16)), RNG.normal(0, 1, (1, 1, 16))
    dots = [float(np.sum(O.rope(q, [m], 10000.0) * O.rope(k, [n], 10000.0)))
            for m, n in ((5, 2), (103, 100), (4003, 4000))]
    assert np.allclose(dots, dots[0], atol=1e-9)                                    # depends on m-n only
    d2 = float(np.sum(O.rope(q, [5], 10000.0) * O.rope(k, [3], 10000.0)))
    assert abs(d2 - dots[0]) > 1e-3                                                 # and does depend on it


def test_rope_complex_formulation():
    """Pair (u[t], u[t+hd/2]) as a complex number times exp(i*pos*base^(-2t/hd))."""
    hd, base = 8, 10000.0
    u = RNG.normal(0, 1, (4, 3, hd))
    pos = np.array([0, 1, 9, 300])
    got = O.rope(u, pos, base)
    for n in range(4):
        for h in range(3):
            for t in range(hd // 2):
                z = complex(u[n, h, t], u[n, h, t + hd // 2]) * complex(
                    math.cos(pos[n] * base ** (-2 * t / hd)), math.sin(pos[n] * base ** (-2 * t / hd)))
                assert abs(got[n, h, t] - z.real) < 1e-12 and abs(got[n, h, t + hd // 2] - z.imag) < 1e-12
    # first pair rotates by exactly `pos` radians (frequency 1), last by pos*base^-(1-2/hd)
    e = np.zeros((1, 1, hd)); e[0, 0, 0] = 1.0
    r = O.rope(e, [2], base)
    assert np.allclose([r[0, 0, 0], r[0, 0, hd // 2]], [math.cos(2.0), math.sin(2.0)], atol=1e-15)


# ---------------------------------------------------------------------------- attention

def _contig_case(B, p, s, Hq, Hkv, hd, blk, peaky=False):
    """Random q and contiguous pools (identity tables) for stand-alone attention."""
    p, s = np.asarray(p), np.asarray(s)
    cu = np.concatenate([[0], np.cumsum(s)]).astype(np.int32)
    need = (p + s + blk - 1) // blk
    tables = np.zeros((B, need.max()), np.int32)
    at = 0
    for b in range(B):
        tables[b, :need[b]] = np.arange(at, at + need[b]); at += need[b]
    q = RNG.normal(0, 4.0 if peaky else 1.0, (cu[-1], Hq, hd))
    kp = O.float_to_bf16(RNG.normal(0, 1, (at, Hkv, blk, hd)))
    vp = O.float_to_bf16(RNG.normal(0, 1, (at, Hkv, blk, hd)))
    return q, kp, vp, p.astype(np.int32), cu, tables


def test_attention_softmax_rows_sum_to_one():
    q, kp, vp, p, cu, tb = _contig_case(2, [9, 3], [4, 6], 4, 2, 8, 4, peaky=True)
    _, probs = O.append_attention(q, kp, vp, p, cu, tb, 4, return_probs=True)
    assert len(probs) == 2 * 4
    for P in probs:
        assert np.all(P >= 0.0) and np.allclose(P.sum(axis=-1), 1.0, atol=1e-12)
    # causal inside the step: query i sees exactly p+i+1 keys
    P0 = probs[0]
    for i in range(4):
        assert np.all(P0[i, 9 + i + 1:] == 0.0) and np.all(P0[i, :9 + i + 1] > 0.0)


def test_attention_matches_torch_sdpa_gqa():
    B, Hq, Hkv, hd, blk = 3, 6, 2, 16, 4
    q, kp, vp, p, cu, tb = _contig_case(B, [10, 0, 7], [5, 3, 1], Hq, Hkv, hd, blk, peaky=True)
    got = O.append_attention(q, kp, vp, p, cu, tb, blk)
    G = Hq // Hkv
    for b in range(B):
        n, s = int(p[b] + cu[b + 1] - cu[b]), int(cu[b + 1] - cu[b])
        K = torch.from_numpy(O.bf16_to_float(kp[tb[b]])).permute(1, 0, 2, 3).reshape(Hkv, -1, hd)[:, :n]
        V = torch.from_numpy(O.bf16_to_float(vp[tb[b]])).permute(1, 0, 2, 3).reshape(Hkv, -1, hd)[:, :n]
        Q = torch.from_numpy(q[cu[b]:cu[b + 1]]).permute(1, 0, 2)                     # [Hq, s, hd]
        mask = torch.ones(s, n, dtype=torch.bool).tril(diagonal=n - s)
        ref = torch.nn.functional.scaled_dot_product_attention(
            Q[None], K.repeat_interleave(G, 0)[None], V.repeat_interleave(G, 0)[None], attn_mask=mask)[0]
        assert np.allclose(got[cu[b]:cu[b + 1]], ref.permute(1, 0, 2).numpy(), atol=1e-12)


def test_attention_closed_forms():
    Hq, Hkv, hd, blk = 2, 1, 8, 4
    # all keys equal -> uniform weights -> output is the mean of the visible values
    q, kp, vp, p, cu, tb = _contig_case(1, [6], [3], Hq, Hkv, hd, blk)
    kp[:] = O.float_to_bf16(np.full(hd, 0.5))[None, None, None, :]
    out = O.append_attention(q, kp, vp, p, cu, tb, blk)
    V = O.bf16_to_float(vp).reshape(-1, hd)
    for i in range(3):
        assert np.allclose(out[i, 0], V[:6 + i + 1].mean(axis=0), atol=1e-12)
    # empty prefix, one token: the only key is itself, output = its value
    q, kp, vp, p, cu, tb = _contig_case(1, [0], [1], Hq, Hkv, hd, blk)
    out = O.append_attention(q, kp, vp, p, cu, tb, blk)
    assert np.allclose(out[0, 0], O.bf16_to_float(vp)[0, 0, 0], atol=0) and np.allclose(out[0, 1], out[0, 0])
    # one dominant key: a planted key aligned with q wins the softmax
    q, kp, vp, p, cu, tb = _contig_case(1, [13], [1], Hq, Hkv, hd, blk)
    q[:] = 0.0; q[0, :, 0] = 64.0
    kf = np.zeros((4, 1, blk, hd)); kf[2, 0, 3, 0] = 8.0                              # position 11
    out = O.append_attention(q, O.float_to_bf16(kf), vp, p, cu, tb, blk)
    assert np.allclose(out[0, 0], O.bf16_to_float(vp)[2, 0, 3], atol=1e-9)


def test_gqa_equals_mha_with_duplicated_kv_heads():
    B, Hq, Hkv, hd, blk = 2, 6, 3, 8, 4
    q, kp, vp, p, cu, tb = _contig_case(B, [5, 9], [4, 2], Hq, Hkv, hd, blk)
    got = O.append_attention(q, kp, vp, p, cu, tb, blk)
    G = Hq // Hkv
    ref = O.append_attention(q, np.repeat(kp, G, axis=1), np.repeat(vp, G, axis=1), p, cu, tb, blk)
    assert np.array_equal(got, ref)
    # and the mapping is h // G, not h % Hkv: zeroing kv head 0 changes q heads 0..G-1 only
    vp2 = vp.copy(); vp2[:, 0] = 0
    diff = np.abs(O.append_attention(q, kp, vp2, p, cu, tb, blk) - got).max(axis=(0, 2))
    assert np.all(diff[:G] > 0) and np.all(diff[G:] == 0)


# --------------------------------------------------------------------------------- MLP

def test_swiglu_against_torch_and_special_cases():
    d, f = 16, 24
    x, wgu, wd = RNG.normal(0, 1, (5, d)), RNG.normal(0, 0.5, (2 * f, d)), RNG.normal(0, 0.5, (d, f))
    xt, g, u = torch.from_numpy(x), torch.from_numpy(wgu[:f]), torch.from_numpy(wgu[f:])
    ref = torch.nn.functional.linear(
        torch.nn.functional.silu(torch.nn.functional.linear(xt, g)) * torch.nn.functional.linear(xt, u),
        torch.from_numpy(wd)).numpy()
    assert np.allclose(O.swiglu_mlp(x, wgu, wd), ref, atol=1e-12)
    assert O.silu(np.array([0.0]))[0] == 0.0 and abs(O.silu(np.array([1.0]))[0] - 1 / (1 + math.exp(-1))) < 1e-15
    assert np.all(O.swiglu_mlp(x, wgu, np.zeros((d, f))) == 0.0)
    # gate and up are not interchangeable
    swapped = np.concatenate([wgu[f:], wgu[:f]])
    assert np.abs(O.swiglu_mlp(x, swapped, wd) - ref).max() > 1e-3


# ------------------------------------------------------------------ whole forward pins

def _torch_full_causal(model: W.ModelShape, weights: W.Weights, ids: np.ndarray):
    """One sequence, no cache, torch fp64 library ops, explicit (n x n) mask.
    K and V pass through bf16 because the cache the method reads from is bf16."""
    Hq, Hkv, hd, d = model.n_q_heads, model.n_kv_heads, model.head_dim, model.d_model
    n = len(ids)
    dd = lambda t: t.double()
    h = torch.nn.functional.embedding(torch.from_numpy(ids.astype(np.int64)), dd(weights.embed))
    t = torch.arange(hd // 2, dtype=torch.float64)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * model.rope_base ** (-2.0 * t / hd)[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]                          # e^{i theta}

    def rope(u):                                                                     # [n, H, hd]
        z = torch.complex(u[..., :hd // 2], u[..., hd // 2:]) * rot
        return torch.cat([z.real, z.imag], dim=-1)

    mask = torch.ones(n, n, dtype=torch.bool).tril()
    for l in range(model.n_layers):
        x = torch.nn.functional.rms_norm(h, (d,), dd(weights.g_attn[l]), eps=model.rms_eps)
        qkv = torch.nn.functional.linear(x, dd(weights.wqkv[l])).view(n, Hq + 2 * Hkv, hd)
        q = rope(qkv[:, :Hq])
        k = rope(qkv[:, Hq:Hq + Hkv]).float().bfloat16().double()
        v = qkv[:, Hq + Hkv:].float().bfloat16().double()
        o = torch.nn.functional.scaled_dot_product_attention(
            q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None], v.permute(1, 0, 2)[None], attn_mask=mask,
            enable_gqa=True)[0].permute(1, 0, 2).reshape(n, Hq * hd)
        h = h + torch.nn.functional.linear(o, dd(weights.wo[l]))
        x = torch.nn.functional.rms_norm(h, (d,), dd(weights.g_mlp[l]), eps=model.rms_eps)
        gu = torch.nn.functional.linear(x, dd(weights.wgu[l]))
        f = model.d_ffn
        h = h + torch.nn.functional.linear(torch.nn.functional.silu(gu[:, :f]) * gu[:, f:], dd(weights.wd[l]))
    return torch.nn.functional.rms_norm(h, (d,), dd(weights.g_final), eps=model.rms_eps).numpy()


def test_append_equals_full_causal_forward():
    """prefill(x) then append(z) == one causal pass over x||z (hidden states of z),
    the latter computed without any cache by torch library routines."""
    batch, weights = small_case()
    m, p, kp, vp, prompt, scores, esc, y = run_prefill_then_step(batch, weights)
    at = 0
    for b in range(batch.batch):
        pl = int(batch.prefix_lens[b])
        ids = np.concatenate([prompt[at:at + pl], batch.token_ids[batch.cu_step_lens[b]:batch.cu_step_lens[b + 1]]])
        at += pl
        ref = _torch_full_causal(SMALL, weights, ids)[pl:]
        got = y[batch.cu_step_lens[b]:batch.cu_step_lens[b + 1]]
        assert np.allclose(got, ref, atol=1e-9, rtol=0), np.abs(got - ref).max()
        # mean-pooled linear head + bias
        s_ref = ref.mean(axis=0) @ weights.w_head.double().numpy() + weights.b_head
        assert abs(scores[b] - s_ref) < 1e-9


def test_append_equals_oracle_prefill_of_concatenation_and_kv():
    """Same statement inside the oracle, including the cache contents."""
    batch, weights = small_case()
    m, p, kp, vp, prompt, scores, esc, y = run_prefill_then_step(batch, weights)
    kp2, vp2 = oracle_pools(*W.make_kv_pools(SMALL_W, batch))
    ids, at = [], 0
    for b in range(batch.batch):
        pl = int(batch.prefix_lens[b])
        ids += [prompt[at:at + pl], batch.token_ids[batch.cu_step_lens[b]:batch.cu_step_lens[b + 1]]]
        at += pl
    tot = batch.prefix_lens + batch.step_lens
    cu = np.concatenate([[0], np.cumsum(tot)]).astype(np.int32)
    yfull = O.prefill(m, p, kp2, vp2, np.concatenate(ids), cu, batch.block_tables)
    for b in range(batch.batch):
        ref = yfull[cu[b] + batch.prefix_lens[b]:cu[b + 1]]
        assert np.allclose(y[batch.cu_step_lens[b]:batch.cu_step_lens[b + 1]], ref, atol=1e-9)
    for l in range(SMALL.n_layers):
        assert np.array_equal(kp[l], kp2[l]) and np.array_equal(vp[l], vp2[l])


def _py_bf16(x: float) -> float:
    """Nearest-even bf16 of a Python float via struct (a route of its own)."""
    (u,) = struct.unpack("<I", struct.pack("<f", x))
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return struct.unpack("<f", struct.pack("<I", u))[0]


def test_brute_force_tiny_pure_python():
    """L1, d8, Hq2, Hkv1, hd4, p3, s2: every sum written out as a Python loop over
    an explicit (p+s) x (p+s) masked score matrix, Python floats (fp64)."""
    ms = W.ModelShape("pin-tiny", 1, 8, 2, 1, 4, 12, 19, kv_block=2)
    wl = W.Workload("pin-tiny", ms, 1, (3, 3), ("fixed", 2, 2), "shuffled", "prefill", 0.0, ("const", 0.0), 3)
    batch = W.make_batch(wl)
    weights = W.make_weights(ms, wl.seed, sigma=0.5, gain_jitter=0.2, b_head=-0.125)
    _, _, _, _, prompt, scores, esc, y = run_prefill_then_step(batch, weights, ms, wl)

    d, Hq, hd, f, n, eps = 8, 2, 4, 12, 5, ms.rms_eps
    fl = lambda t: t.double().tolist()
    E, Wqkv, Wo, Wgu, Wd = fl(weights.embed), fl(weights.wqkv[0]), fl(weights.wo[0]), fl(weights.wgu[0]), fl(weights.wd[0])
    ga, gm, gf, wh = fl(weights.g_attn[0]), fl(weights.g_mlp[0]), fl(weights.g_final), fl(weights.w_head)
    ids = list(prompt) + list(batch.token_ids)

    def norm(row, g):
        r = math.sqrt(sum(v * v for v in row) / d + eps)
        return [row[c] / r * g[c] for c in range(d)]

    def matvec(Wm, x):
        return [sum(Wm[o][c] * x[c] for c in range(len(x))) for o in range(len(Wm))]

    def rot(vec, pos):
        out = list(vec)
        for t in range(hd // 2):
            th = pos * ms.rope_base ** (-2.0 * t / hd)
            a, b = vec[t], vec[t + hd // 2]
            out[t], out[t + hd // 2] = a * math.cos(th) - b * math.sin(th), b * math.cos(th) + a * math.sin(th)
        return out

    h = [list(E[i]) for i in ids]
    xs = [norm(r, ga) for r in h]
    qkv = [matvec(Wqkv, x) for x in xs]
    q = [[rot(qkv[i][hh * hd:(hh + 1) * hd], i) for hh in range(Hq)] for i in range(n)]
    k = [[_py_bf16(v) for v in rot(qkv[i][Hq * hd:(Hq + 1) * hd], i)] for i in range(n)]
    v = [[_py_bf16(c) for c in qkv[i][(Hq + 1) * hd:(Hq + 2) * hd]] for i in range(n)]
    attn = [[0.0] * (Hq * hd) for _ in range(n)]
    for hh in range(Hq):
        S = [[sum(q[i][hh][c] * k[j][c] for c in range(hd)) / math.sqrt(hd) if j <= i else None
              for j in range(n)] for i in range(n)]
        for i in range(n):
            mx = max(s for s in S[i] if s is not None)
            e = [math.exp(s - mx) if s is not None else 0.0 for s in S[i]]
            z = sum(e)
            for c in range(hd):
                attn[i][hh * hd + c] = sum(e[j] / z * v[j][c] for j in range(n))
    for i in range(n):
        o = matvec(Wo, attn[i])
        h[i] = [h[i][c] + o[c] for c in range(d)]
        x = norm(h[i], gm)
        gu = matvec(Wgu, x)
        act = [gu[c] / (1.0 + math.exp(-gu[c])) * gu[f + c] for c in range(f)]
        dn = matvec(Wd, act)
        h[i] = [h[i][c] + dn[c] for c in range(d)]
    yy = [norm(r, gf) for r in h]
    for i in range(2):
        assert np.allclose(y[i], yy[3 + i], atol=1e-10), (y[i], yy[3 + i])
    sc = sum(wh[c] * (yy[3][c] + yy[4][c]) / 2 for c in range(d)) + weights.b_head
    assert abs(scores[0] - sc) < 1e-10
    assert esc[0] == (0 if np.float32(sc) <= np.float32(0.0) else 1)


def test_paged_equals_contiguous_bit_identical():
    batch, weights = small_case()
    _, _, kp, vp, _, scores, _, y = run_prefill_then_step(batch, weights)
    # renumber the pool blocks with another permutation and move the filler along
    perm = np.random.default_rng(5).permutation(batch.n_blocks).astype(np.int32)
    b2 = W.Batch(batch.prefix_lens, batch.cu_step_lens, perm[batch.block_tables], batch.token_ids,
                 batch.n_blocks, batch.kv_block, batch.tau)
    m, p = oracle_model(SMALL), oracle_params(weights)
    k0, v0 = oracle_pools(*W.make_kv_pools(SMALL_W, batch))
    kq = [np.empty_like(a) for a in k0]; vq = [np.empty_like(a) for a in v0]
    for l in range(SMALL.n_layers):
        kq[l][perm] = k0[l]; vq[l][perm] = v0[l]
    prompt = W.prompt_token_ids(SMALL_W, batch)
    cu_p = np.concatenate([[0], np.cumsum(batch.prefix_lens)]).astype(np.int32)
    O.prefill(m, p, kq, vq, prompt, cu_p, b2.block_tables)
    s2, _, y2 = O.score_steps(m, p, kq, vq, b2.token_ids, b2.prefix_lens, b2.cu_step_lens, b2.block_tables, 0.0)
    assert np.array_equal(y, y2) and np.array_equal(scores, s2)
    for l in range(SMALL.n_layers):
        assert np.array_equal(kq[l][perm], kp[l]) and np.array_equal(vq[l][perm], vp[l])


def test_scoring_leaves_prefix_and_spare_blocks_untouched_and_is_idempotent():
    batch, weights = small_case()
    m, p = oracle_model(SMALL), oracle_params(weights)
    kp, vp = oracle_pools(*W.make_kv_pools(SMALL_W, batch))
    prompt = W.prompt_token_ids(SMALL_W, batch)
    cu_p = np.concatenate([[0], np.cumsum(batch.prefix_lens)]).astype(np.int32)
    O.prefill(m, p, kp, vp, prompt, cu_p, batch.block_tables)
    before = [a.copy() for a in kp + vp]
    args = (batch.token_ids, batch.prefix_lens, batch.cu_step_lens, batch.block_tables, batch.tau)
    s1, _, y1 = O.score_steps(m, p, kp, vp, *args)
    step_slots = set(O.slot_mapping(batch.prefix_lens, batch.cu_step_lens, batch.block_tables, 4).tolist())
    for a, b4 in zip(kp + vp, before):
        flat_a = a.transpose(0, 2, 1, 3).reshape(-1, a.shape[1], a.shape[3])
        flat_b = b4.transpose(0, 2, 1, 3).reshape(-1, a.shape[1], a.shape[3])
        changed = {i for i in range(flat_a.shape[0]) if not np.array_equal(flat_a[i], flat_b[i])}
        assert changed <= step_slots and len(changed) == len(step_slots)
    s2, _, y2 = O.score_steps(m, p, kp, vp, *args)
    assert np.array_equal(s1, s2) and np.array_equal(y1, y2)


def test_zero_projections_reduce_to_identity():
    batch, weights = small_case(gain_jitter=0.0)
    for l in range(SMALL.n_layers):
        weights.wo[l].zero_(); weights.wd[l].zero_()
    _, p, _, _, _, _, _, y = run_prefill_then_step(batch, weights)
    ref = O.rmsnorm(O.embed(p.embed, batch.token_ids), np.ones(SMALL.d_model), SMALL.rms_eps)
    assert np.allclose(y, ref, atol=1e-12)


def test_decoder_layers_is_the_forward_without_its_ends_and_ranges_compose():
    """decoder_layers referees the per-layer GPU checks, so it is pinned here: over all layers it is
    forward() before the final norm (same bits, same cache); the stream it keeps after layer l is the
    one a model cut off after l + 1 layers normalises; consecutive ranges compose bit for bit."""
    from dataclasses import replace
    deep = replace(SMALL, n_layers=3)
    wl = replace(SMALL_W, model=deep)
    batch = W.make_batch(wl)
    weights = W.make_weights(deep, wl.seed, sigma=0.3, gain_jitter=0.1)
    m, p = oracle_model(deep), oracle_params(weights)
    pools = lambda: oracle_pools(*W.make_kv_pools(wl, batch))
    args = (batch.prefix_lens, batch.cu_step_lens, batch.block_tables)
    kp0, vp0 = pools()
    y = O.forward(m, p, kp0, vp0, batch.token_ids, *args)
    kp1, vp1 = pools()
    h0 = O.embed(p.embed, batch.token_ids)
    keep = []
    h = O.decoder_layers(m, p, kp1, vp1, h0, 0, 3, *args, keep=keep)
    assert len(keep) == 3 and keep[-1] is h
    assert np.array_equal(O.rmsnorm(h, p.g_final, deep.rms_eps), y)
    for l in range(3):
        assert np.array_equal(kp0[l], kp1[l]) and np.array_equal(vp0[l], vp1[l])
    # the kept stream after layer l, against a model that ends there
    for l in range(3):
        cut = replace(deep, n_layers=l + 1)
        kpc, vpc = pools()
        yc = O.forward(oracle_model(cut), p, kpc, vpc, batch.token_ids, *args)
        assert np.array_equal(O.rmsnorm(keep[l], p.g_final, deep.rms_eps), yc)
        assert not np.array_equal(keep[l], keep[l - 1] if l else h0)
    # [0, 1) then [1, 3) is [0, 3); a range touches only its own layers' cache
    kp2, vp2 = pools()
    fresh = [a.copy() for a in kp2]
    mid = O.decoder_layers(m, p, kp2, vp2, h0, 0, 1, *args)
    assert np.array_equal(mid, keep[0])
    assert np.array_equal(kp2[1], fresh[1]) and np.array_equal(kp2[2], fresh[2]) and not np.array_equal(kp2[0], fresh[0])
    end = O.decoder_layers(m, p, kp2, vp2, mid, 1, 3, *args)
    assert np.array_equal(end, h)
    for l in range(3):
        assert np.array_equal(kp2[l], kp1[l]) and np.array_equal(vp2[l], vp1[l])
    # an empty range is the identity
    assert np.array_equal(O.decoder_layers(m, p, kp2, vp2, h0, 2, 2, *args), h0)


def test_fp32_weights_are_the_bf16_values():
    """Params given as widened floats or as bf16 bits are the same model."""
    batch, weights = small_case()
    _, p, _, _, _, s1, _, _ = run_prefill_then_step(batch, weights)
    assert p.wqkv[0].dtype == np.uint16
    assert np.array_equal(O.as_float(p.wqkv[0]), weights.wqkv[0].double().numpy())


# ------------------------------------------------------------------- pooling and head

def test_router_head_closed_forms():
    cu = np.array([0, 3, 4, 9], np.int32)
    y = RNG.normal(0, 1, (9, 6)); w = RNG.normal(0, 1, 6)
    const = np.tile(RNG.normal(0, 1, 6), (9, 1))
    assert np.allclose(O.router_scores(const, cu, w, 0.5), const[0] @ w + 0.5, atol=1e-12)
    assert np.all(O.router_scores(y, cu, np.zeros(6), -2.0) == -2.0)                  # w = 0 -> bias
    mean, last = O.router_scores(y, cu, w, 0.0, "mean"), O.router_scores(y, cu, w, 0.0, "last")
    assert mean[1] == last[1]                                                        # one-token step
    assert np.allclose(last, [y[2] @ w, y[3] @ w, y[8] @ w], atol=1e-12)
    assert np.allclose(mean[2], np.mean(y[4:9] @ w), atol=1e-12)                      # head is linear
    assert abs(mean[0] - last[0]) > 1e-6


def test_two_class_head_is_the_logistic_of_the_folded_linear_head():
    """Section 4.2 ('Training'): a two-way classification head.  Its class-1 probability depends only on
    the logit difference, so it must equal the logistic function of the linear head with w = w_1 - w_0,
    c = c_1 - c_0; thresholding the probability at tau_p is thresholding that linear score at
    ln(tau_p / (1 - tau_p)) (0.5 <-> 0)."""
    cu = np.array([0, 3, 4, 9], np.int32)
    y = RNG.normal(0, 1, (9, 6)); w2 = RNG.normal(0, 1, (2, 6))
    for mode in ("mean", "last"):
        p = O.router_scores(y, cu, w2, 0.3, mode)
        z = O.router_scores(y, cu, w2[1] - w2[0], 0.3, mode)
        assert np.allclose(p, 1.0 / (1.0 + np.exp(-z)), atol=1e-14)
        assert np.all((p > 0) & (p < 1))
        for tau_p in (0.2, 0.5, 0.9):
            assert np.array_equal(O.route(p, tau_p), O.route(z, np.log(tau_p / (1 - tau_p))))
    # identical rows: the classes cannot be told apart; swapping the rows mirrors the probability
    assert np.allclose(O.router_scores(y, cu, np.stack([w2[0], w2[0]]), 0.0), 0.5, atol=1e-15)
    assert np.allclose(O.router_scores(y, cu, w2[::-1].copy(), -0.3), 1.0 - O.router_scores(y, cu, w2, 0.3), atol=1e-14)
    # large logit differences saturate without overflow
    big = O.router_scores(np.full((9, 6), 50.0), cu, np.stack([np.zeros(6), np.full(6, 20.0)]), 0.0)
    assert np.all(big == 1.0) and np.all(np.isfinite(big))


# --------------------------------------------------------------------------- decision

def test_route_tie_nan_and_sense():
    s = np.array([0.25, 0.5, 0.75, np.nan, -np.inf, np.inf], np.float32)
    # Alg. 1: accept iff y_hat <= tau; equality accepts; NaN escalates
    assert O.route(s, 0.5).tolist() == [0, 0, 1, 1, 0, 1]
    # RSD (Section 3.1): accept iff s_d > tau, the opposite sense; equality rejects
    assert O.route(s, 0.5, "accept_if_gt").tolist() == [1, 1, 0, 1, 1, 0]
    # fp32 decision: a score that differs from tau only beyond fp32 precision ties
    assert O.route(np.array([0.1 + 1e-12]), np.float32(0.1)).tolist() == [0]


@pytest.mark.parametrize("n", [1, 7, 64])
def test_route_theorem_b1_top_k_and_monotone(n):
    """Theorem B.1: with Delta_(k) > tau >= Delta_(k+1) the threshold policy
    escalates exactly the k largest entries; escalations are monotone in tau."""
    delta = np.random.default_rng(n).normal(0, 1, n).astype(np.float32)
    order = np.argsort(-delta, kind="stable")
    srt = delta[order]
    seen = []
    for k in range(n + 1):
        hi = srt[k - 1] if k > 0 else np.float32(np.inf)
        lo = srt[k] if k < n else np.float32(-np.inf)
        tau = lo if np.isfinite(lo) else np.float32(srt[-1] - 1)                    # tau = Delta_(k+1) is allowed
        a = O.route(delta, tau)
        assert a.sum() == k and set(np.nonzero(a)[0]) == set(order[:k])
        if np.isfinite(hi) and np.isfinite(lo) and hi > lo:
            mid = np.float32((np.float64(hi) + np.float64(lo)) / 2)
            if lo <= mid < hi:
                assert np.array_equal(O.route(delta, mid), a)
        seen.append((float(tau), int(a.sum())))
    seen.sort()
    assert all(c0 >= c1 for (_, c0), (_, c1) in zip(seen, seen[1:]))                 # non-increasing in tau
    # budget B with the k = min(B, #positive) rule: the optimum of sum a_i*Delta_i
    B = max(1, n // 3)
    k = min(B, int((delta > 0).sum()))
    tau = srt[k] if k < n else np.float32(srt[-1] - 1)
    a = O.route(delta, max(tau, np.float32(0.0)) if k < B else tau)
    best = np.sort(delta[delta > 0])[::-1][:B].sum()
    assert np.isclose(float((a * delta).sum()), float(best), rtol=1e-6)


def test_route_zero_waste_corollary_and_realized_score():
    """Corollary B.3: at tau = 0 on Delta no escalated step has s_t <= s_d; and
    S(a) = s_d + a*Delta (Definition 4.2) is maximal step-wise under that policy."""
    r = np.random.default_rng(11)
    s_d, s_t = r.normal(0, 1, 200).astype(np.float32), r.normal(0, 1, 200).astype(np.float32)
    s_t[:20] = s_d[:20]                                                              # ties: Delta = 0 accepts
    delta = O.advantage(s_t, s_d)
    a = O.route(delta, 0.0)
    assert not np.any((a == 1) & (s_t <= s_d)) and np.all(a[:20] == 0)
    assert np.allclose(O.realized_score(s_d, s_t, a), np.maximum(s_d, s_t))
    assert np.allclose(O.realized_score(s_d, s_t, a), s_d + a * delta)


@pytest.mark.parametrize("n,seed", [(1, 0), (5, 1), (9, 2), (10, 3)])
def test_budget_threshold_attains_the_brute_force_optimum(n, seed):
    """Theorem B.1 by exhaustion: for every budget the threshold policy's value equals the
    maximum of sum a_i*Delta_i over all 2^n policies with at most `budget` escalations."""
    import itertools
    delta = np.random.default_rng(seed).normal(0.2, 1, n).astype(np.float32)
    for budget in range(n + 2):
        best = max(sum(d for d, a in zip(delta.astype(np.float64), bits) if a)
                   for bits in itertools.product((0, 1), repeat=n) if sum(bits) <= budget)
        tau = O.budget_threshold(delta, budget)
        a = O.route(delta, tau)
        assert a.sum() <= budget and tau >= 0
        assert np.isclose(float((a * delta.astype(np.float64)).sum()), best, rtol=1e-6, atol=1e-7)
    # entries that are NaN escalate whatever tau is and use up budget first
    d = np.array([0.5, np.nan, 2.0, 1.0, np.nan], np.float32)
    assert O.budget_threshold(d, 1) == float("inf") and O.route(d, np.inf).tolist() == [0, 1, 0, 0, 1]
    assert O.budget_threshold(d, 3) == 1.0 and O.route(d, 1.0).sum() == 3
    assert O.budget_threshold(d, 9) == 0.0


def test_choose_token_greedy_and_inversion_sampling():
    r = np.random.default_rng(3)
    logits = r.normal(0, 2, 50)
    assert O.choose_token(logits) == int(np.argmax(logits)) == O.choose_token(logits, 0.0)
    assert O.choose_token(np.array([1.0, 3.0, 3.0, 2.0])) == 1                  # first index of the maximum
    # inversion: monotone in u, u = 0 gives token 0, and the frequencies over a fine grid of u are
    # the softmax probabilities (torch library softmax as the independent formulation)
    T = 0.7
    us = (np.arange(200000) + 0.5) / 200000
    ks = np.array([O.choose_token(logits[:8], T, u) for u in us[::40]])
    assert np.all(np.diff(ks) >= 0) and O.choose_token(logits[:8], T, 0.0) == 0
    freq = np.bincount(ks, minlength=8) / ks.size
    p = torch.softmax(torch.tensor(logits[:8], dtype=torch.float64) / T, 0).numpy()
    assert np.abs(freq - p).max() < 2e-3
    # temperature -> 0 approaches greedy; a very high temperature approaches uniform
    assert O.choose_token(logits, 1e-3, 0.5) == int(np.argmax(logits))
    assert O.choose_token(logits, 1e6, 0.999) == 49


def test_first_stop_and_lm_logits():
    assert O.first_stop([5, 6, 9, 7, 8], sep=9, eos=8) == (3, False)
    assert O.first_stop([5, 8, 9], sep=9, eos=8) == (2, True)
    assert O.first_stop([5, 6], sep=9, eos=8) == (2, False) and O.first_stop([], 9, 8) == (0, False)
    h = np.array([[1.0, 2.0], [0.5, -1.0]])
    w = O.float_to_bf16(np.array([[1.0, 0.0], [0.0, 1.0], [2.0, 2.0]]))
    assert np.array_equal(O.lm_logits(h, w), np.array([[1.0, 2.0, 6.0], [0.5, -1.0, -1.0]]))


def test_arbitrage_inference_follows_algorithm_1():
    SEP, EOS = 1, 2
    calls = []
    def draft(x):
        calls.append(("d", len(x)))
        return [10 + len(x), SEP]
    def target(x):
        calls.append(("t", len(x)))
        return [90, EOS] if len(x) >= 11 else [50 + len(x), 51, SEP]
    # y_hat = 0.5 exactly at the second step (a tie accepts), above tau at the third, below otherwise
    scores = iter([0.1, 0.5, 0.9, 0.2, 0.9])
    def router(x, z):
        calls.append(("r", len(x), tuple(z)))
        return next(scores)
    x, log = O.arbitrage_inference([7, 8 + 1], draft, router, target, tau=0.5, eos=EOS, max_steps=10)
    # steps: accept, accept (tie), escalate (target step of 3 tokens from the same prefix), accept, escalate -> eos
    assert [e for _, e in log] == [False, False, True, False, True]
    assert x == [7, 9, 12, SEP, 14, SEP, 56, 51, SEP, 19, SEP, 90, EOS]
    # the target regenerates from the same prefix the draft saw; the router sees the draft's step
    assert ("d", 6) in calls and ("t", 6) in calls and ("r", 6, (16, SEP)) in calls
    # stops at eos without another draft call, and at max_steps
    assert calls[-1][0] == "t" and len(log) == 5
    x2, log2 = O.arbitrage_inference([7], draft, lambda x, z: 0.0, target, tau=0.5, eos=EOS, max_steps=3)
    assert len(log2) == 3 and x2 == [7, 11, SEP, 13, SEP, 15, SEP]
    assert O.arbitrage_inference([7, EOS], draft, router, target, 0.5, EOS, 5) == ([7, EOS], [])


def test_w4_quantization_definition():
    r = np.random.default_rng(12)
    w = O.float_to_bf16(r.normal(0, 0.02, (6, 384)))
    w[2, 128:256] = 0                                                    # a group of zeros: scale 0, q 0
    q, sb = O.w4_quantize(w)
    wf, s = O.bf16_to_float(w), O.bf16_to_float(sb)
    assert q.dtype == np.int8 and q.min() >= -8 and q.max() <= 7 and sb.shape == (6, 3)
    assert np.all(q[2, 128:256] == 0) and s[2, 1] == 0
    wd = O.w4_dequantize(q, sb)
    g = lambda a: a.reshape(6, 3, 128)
    # the scale is max|w|/7 to bf16 precision; the error of an unclipped entry is at most half a step
    assert np.allclose(s, np.abs(g(wf)).max(2) / 7, rtol=2 ** -8)
    unclipped = np.abs(g(wf)) <= 7 * s[:, :, None]
    assert np.all(np.abs(g(wd) - g(wf))[unclipped] <= 0.5 * np.repeat(s[:, :, None], 128, 2)[unclipped] * (1 + 1e-6))
    # the largest entry of a group lands on +-7 (or +-8 where the bf16 rounding of the scale went down)
    big = np.abs(g(q)).max(2)
    assert np.all((big[s > 0] == 7) | (big[s > 0] == 8))
    # integers times the scale are fixed points
    again, sb2 = O.w4_quantize(O.float_to_bf16(7 * np.repeat(s, 128, 1) * np.sign(r.normal(size=(6, 384)))))
    assert np.array_equal(sb2, sb) and np.all(np.abs(again[np.repeat(s, 128, 1) > 0]) == 7)
    # packing: word i holds q[8i .. 8i+7] + 8, the even ones in nibbles 0..3, the odd ones in nibbles 4..7
    p = O.w4_pack(q)
    assert p.dtype == np.uint32 and p.shape == (6, 48)
    for (n, k) in ((0, 0), (0, 1), (3, 77), (3, 78), (5, 382), (5, 383)):
        nibble = (k % 8) // 2 + 4 * (k % 2)
        assert (int(p[n, k // 8]) >> (4 * nibble)) & 15 == int(q[n, k]) + 8
    one = np.zeros((1, 128), np.int8); one[0, :8] = [-8, -7, -6, -5, -4, -3, -2, -1]
    assert int(O.w4_pack(one)[0, 0]) == 0x75316420


def test_w3_quantization_is_the_same_rule_with_levels_minus4_to_3():
    r = np.random.default_rng(13)
    w = O.float_to_bf16(r.normal(0, 0.02, (5, 256)))
    w[1, :128] = 0
    q, sb = O.w4_quantize(w, bits=3)
    wf, s = O.bf16_to_float(w), O.bf16_to_float(sb)
    g = lambda a: a.reshape(5, 2, 128)
    assert q.dtype == np.int8 and q.min() >= -4 and q.max() <= 3 and np.all(q[1, :128] == 0) and s[1, 0] == 0
    assert np.allclose(s, np.abs(g(wf)).max(2) / 3, rtol=2 ** -8)
    wd = O.w4_dequantize(q, sb)
    unclipped = np.abs(g(wf)) <= 3 * s[:, :, None]
    assert np.all(np.abs(g(wd) - g(wf))[unclipped] <= 0.5 * np.repeat(s[:, :, None], 128, 2)[unclipped] * (1 + 1e-6))
    big = np.abs(g(q)).max(2)
    assert np.all((big[s > 0] == 3) | (big[s > 0] == 4))
    # eight levels are coarser than sixteen: on the same weights the 3-bit error is the larger one (about 7/3 of it)
    q4, sb4 = O.w4_quantize(w)
    e3 = np.sqrt(np.mean((wd - wf) ** 2)); e4 = np.sqrt(np.mean((O.w4_dequantize(q4, sb4) - wf) ** 2))
    assert 1.8 < e3 / e4 < 2.9
    # the nibble format holds them unchanged
    p = O.w4_pack(q)
    assert (int(p[4, 31]) >> 28) & 15 == int(q[4, 255]) + 8 and (int(p[4, 31]) >> 12) & 15 == int(q[4, 254]) + 8
    with pytest.raises(ValueError):
        O.w4_quantize(w, bits=5)


# ----------------------------------------------------------------------- stored values

def _golden(name):
    import os
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)


def test_route_rule_table_from_the_paper():
    rows = [l.split() for l in open(_golden("route_rule.txt")) if l.strip() and not l.startswith("#")]
    for score, tau, arb, rsd in rows:
        assert O.route([float(score)], float(tau))[0] == int(arb)
        assert O.route([float(score)], float(tau), "accept_if_gt")[0] == int(rsd)


def test_oracle_small_case_has_not_drifted():
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_golden", _golden("make_golden.py"))
    mod = importlib.util.module_from_spec(spec); spec.loader.exec_module(mod)
    batch, scores, esc, y = mod.compute()
    want = {l.split()[0]: l.split()[1:] for l in open(_golden("oracle_small_case.txt")) if not l.startswith("#")}
    assert list(map(int, want["prefix_lens"])) == batch.prefix_lens.tolist()
    assert np.allclose(scores, list(map(float, want["scores"])), rtol=1e-9, atol=1e-11)
    assert esc.tolist() == list(map(int, want["escalate"]))
    assert np.allclose(y[0, :4], list(map(float, want["hidden_first_row_head"])), rtol=1e-9, atol=1e-11)
    assert np.allclose(y[-1, -4:], list(map(float, want["hidden_last_row_tail"])), rtol=1e-9, atol=1e-11)
