"""Benchmark of the step-scoring hot path on one MI355X.

A step = one arb_score_steps call (embedding, L transformer layers of
append-attention + projections, final norm, pooled router head, threshold) over
one batch of a synthetic workload, inputs resident in HBM.  The headline line is
the 1.5B-router-shaped workload C2 (16 sequences, 2048-token cached prefix,
64-token drafted step); `per_config` carries the same measurements for every
full-size workload (C2..C5): step time, scored step-tokens/s, append-attention
GB/s and its fraction of HBM peak, per-projection and aggregate GEMM TFLOP/s and
their fraction of the bf16 MFMA peak, the whole step against its roofline, and
the CPU oracle timed on a bounded sample.  Prints one JSON line.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# Counter runs of the dominant kernel on workload C2 (profiles/score_steps_C2_hbm_traffic.txt): scaled
# FETCH_SIZE + WRITE_SIZE bytes per launch, and the SHA-256 of the csrc/gemm.hip they were taken with.
COUNTED_GATE_UP_BYTES = 75791396 + 16777216
COUNTED_GEMM_SHA256 = "b92d31b84caa34adf6078b6498e96b8c33086020f1e92ebbd1713c867cefe0f5"

# Which sequences the CPU oracle recomputes per workload (the rungs of the stated ladder): the whole batch
# where that takes seconds, else a seeded sub-batch at full depth that includes the extremes.
CPU_SAMPLE = {"C2": "all", "C3": "all", "C4": 8, "C5": 4}


def _pick(name, batch):
    import numpy as np
    kind = CPU_SAMPLE.get(name, "all")
    if kind == "all":
        return list(range(batch.batch))
    if name == "C5":     # shortest and longest prefix of each step kind (even: 1 token, odd: 64)
        dec, big = np.arange(0, batch.batch, 2), np.arange(1, batch.batch, 2)
        return sorted({int(dec[np.argmin(batch.prefix_lens[dec])]), int(dec[np.argmax(batch.prefix_lens[dec])]),
                       int(big[np.argmin(batch.prefix_lens[big])]), int(big[np.argmax(batch.prefix_lens[big])])})
    pick = {int(np.argmin(batch.prefix_lens)), int(np.argmax(batch.prefix_lens)),
            int(np.argmin(batch.step_lens)), int(np.argmax(batch.step_lens))}
    for b in np.random.default_rng(0).permutation(batch.batch):
        if len(pick) >= kind:
            break
        pick.add(int(b))
    return sorted(pick)


def cpu_baseline(name, w, sess, layers: int):
    """The CPU oracle, as it stands, on a bounded sample of the workload: the sequences of _pick through
    the first `layers` layers (all of them by default) plus final norm and head; the time is scaled to
    full depth when fewer layers ran.  The cache blocks those sequences reference are copied from the
    device as bf16 bit patterns."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info

    import workloads as W
    from helpers import oracle_model, oracle_params
    from oracle import arb_oracle as O

    batch, L = sess.batch, w.model.n_layers
    pick = _pick(name, batch)
    sub = batch.select(pick)
    need = (sub.prefix_lens + sub.step_lens + 15) // 16
    used = np.concatenate([sub.block_tables[i, :need[i]] for i in range(sub.batch)])
    remap = -np.ones(batch.n_blocks, np.int64); remap[used] = np.arange(len(used))
    tables = np.where(np.arange(sub.block_tables.shape[1])[None, :] < need[:, None], remap[sub.block_tables], 0)
    idx = torch.as_tensor(used, dtype=torch.int64, device="cuda")
    kp = [W.bf16_bits(sess.kv.k_pools[l][idx]).copy() for l in range(layers)]
    vp = [W.bf16_bits(sess.kv.v_pools[l][idx]).copy() for l in range(layers)]
    wt = sess.weights
    cpu = lambda t: t.cpu()
    weights = W.Weights(cpu(wt.embed), [cpu(t) for t in wt.wqkv[:layers]], [cpu(t) for t in wt.wo[:layers]],
                        [cpu(t) for t in wt.wgu[:layers]], [cpu(t) for t in wt.wd[:layers]],
                        [cpu(t) for t in wt.g_attn[:layers]], [cpu(t) for t in wt.g_mlp[:layers]], cpu(wt.g_final),
                        cpu(wt.w_head), wt.b_head)
    m, p = oracle_model(W.scaled(w, n_layers=layers).model), oracle_params(weights)
    t0 = time.perf_counter()
    y = O.forward(m, p, kp, vp, sub.token_ids, sub.prefix_lens, sub.cu_step_lens, tables)
    if w.model.has_router_head:
        O.route(O.router_scores(y, sub.cu_step_lens, p.w_head, p.b_head), batch.tau)
    dt = time.perf_counter() - t0
    threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    full = dt * L / layers
    what = f"all {batch.batch} sequences" if len(pick) == batch.batch else \
        f"{len(pick)} of {batch.batch} sequences (shortest/longest prefix and step among them)"
    depth = f"all {L} layers" if layers == L else f"the first {layers} of {L} layers, time x {L}/{layers}"
    return {"value": sub.total_tokens / full, "unit": "scored step-tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{what}, {sub.total_tokens} step tokens against {int(sub.prefix_lens.sum())} cached tokens, "
                      f"{depth}, + final norm and head: {dt:.1f} s"}


STAGES = ("qkv", "attention", "oproj", "gate_up", "down", "norm", "rope_append")


def run_config(name, steps, warmup, cpu_layers, copy_probe_mib=0, stage_reps=3):
    """Sets one workload up on the device, times `steps` calls after `warmup`, then (outside the timed
    region) times every stage with the library's event hook and runs the CPU sample."""
    import torch

    import harness
    import paper_2512_05033_amd as A
    import workloads as W

    w = W.ALL[name]
    sess = harness.setup(w, "cuda")
    batch, model, m = sess.batch, sess.model, w.model
    T, L, d, F = batch.total_tokens, m.n_layers, m.d_model, m.d_ffn
    head = m.has_router_head
    scores = torch.empty(batch.batch, dtype=torch.float32, device="cuda") if head else None
    esc = torch.empty(batch.batch, dtype=torch.uint8, device="cuda") if head else None
    hidden = torch.empty(T, d, dtype=torch.bfloat16, device="cuda")

    def step():
        A.arb_score_steps(model, sess.kv, sess.dbatch, batch.tau, ws=sess.ws, scores=scores, escalate=esc,
                          hidden=hidden)

    if copy_probe_mib > 0:
        src = torch.arange(copy_probe_mib << 18, dtype=torch.float32, device="cuda")   # 4 bytes each
        torch.empty_like(src).copy_(src)
        del src
    for _ in range(warmup):
        step()
    # The gate/up projection's dominant kernel is bracketed by HIP events inside the library, on the stream
    # it runs on, during the timed steps: the kernel with the SwiGLU epilogue, or, where the projection is
    # launched as two kernels, the 256x256-tile kernel that does most of its columns.
    large_cols = A.arb_gemm_large_tile_columns(T, F, d, A.ARB_EPI_SWIGLU_BF16)
    if large_cols > 0:
        gu_stage, gu_features = A.ARB_STAGE_GATE_UP_LARGE, large_cols * 128
        gu_kernel = f"gemm256_kernel<SWIGLU, K-blocked weights> (gate/up projection, features [0, {gu_features}) of {F} in 256x256 tiles)"
    else:
        gu_stage, gu_features = A.ARB_STAGE_GATE_UP, F
        gu_kernel = "gemm_kernel<SWIGLU> (gate/up projection, 128x128 tiles)"
    timer = A.StageTimer(model, gu_stage, steps * L)
    timer.arm()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    n = timer.disarm()
    gu_ms = timer.durations_ms(n)
    timer.close()
    ms_per_step = dt / steps * 1e3
    gu_avg_ms = sum(gu_ms) / len(gu_ms)
    gu_flops = 2.0 * T * (2 * gu_features) * d                            # per launch of that kernel
    gu_achieved = gu_flops / (gu_avg_ms * 1e-3) / 1e12

    # per-stage times: extra passes, outside the timed region
    ids = {"qkv": A.ARB_STAGE_QKV, "attention": A.ARB_STAGE_ATTENTION, "oproj": A.ARB_STAGE_OPROJ,
           "gate_up": A.ARB_STAGE_GATE_UP, "down": A.ARB_STAGE_DOWN, "norm": A.ARB_STAGE_NORM,
           "rope_append": A.ARB_STAGE_ROPE_APPEND}
    reps, stage_ms = max(stage_reps, 1), {}
    for sname in STAGES if stage_reps > 0 else ():
        t = A.StageTimer(model, ids[sname], reps * L)
        t.arm()
        for _ in range(reps):
            step()
        torch.cuda.synchronize()
        dur = t.durations_ms(t.disarm())
        t.close()
        stage_ms[sname] = sum(dur) / reps
    if stage_reps <= 0:        # counter runs: the timed steps only
        model.close()
        return {"workload": w.name, "layers": L, "d_model": d, "batch": batch.batch, "step_tokens": T,
                "prefix_tokens": int(batch.prefix_lens.sum()), "kv": f"paged-16 {w.tables}", "ms_per_step": ms_per_step,
                "step_tokens_per_s": T / (ms_per_step * 1e-3),
                "gemm": {"dominant_kernel": {"kernel": gu_kernel, "avg_launch_ms": gu_avg_ms, "launches": n,
                                             "flops_per_launch": gu_flops, "TFLOPs": gu_achieved,
                                             "mfma_frac": gu_achieved / PEAK_BF16_TFLOPS}}}
    # algorithmic work of one layer
    ctx = (batch.prefix_lens + batch.step_lens).astype(float)
    s, p = batch.step_lens.astype(float), batch.prefix_lens.astype(float)
    kv_bytes = float((ctx * 2 * m.n_kv_heads * m.head_dim * 2).sum())
    qo_bytes = 2.0 * T * m.n_q_heads * m.head_dim * 2
    attn_flops = float((4 * m.n_q_heads * m.head_dim * (s * p + s * (s + 1) / 2)).sum())
    gemm_flops = {"qkv": 2.0 * T * m.qkv_rows * d, "oproj": 2.0 * T * d * m.n_q_heads * m.head_dim,
                  "gate_up": 2.0 * T * 2 * F * d, "down": 2.0 * T * d * F}
    weight_bytes = 2.0 * m.params_per_layer
    attn_s = stage_ms["attention"] / L * 1e-3
    attn_bound_s = max((kv_bytes + qo_bytes) / (PEAK_HBM_GBS * 1e9), attn_flops / (PEAK_BF16_TFLOPS * 1e12))
    gemm_s = sum(stage_ms[k] for k in gemm_flops) / L * 1e-3
    gemm_bound_s = max(sum(gemm_flops.values()) / (PEAK_BF16_TFLOPS * 1e12), weight_bytes / (PEAK_HBM_GBS * 1e9))
    roof_ms = (attn_bound_s + gemm_bound_s) * L * 1e3
    entry = {
        "workload": w.name, "layers": L, "d_model": d, "batch": batch.batch, "step_tokens": T,
        "prefix_tokens": int(batch.prefix_lens.sum()), "kv": f"paged-16 {w.tables}", "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "step_tokens_per_s": T / (ms_per_step * 1e-3),
        "step_roofline": {"ms": roof_ms, "frac": roof_ms / ms_per_step,
                          "what": "per layer max(GEMM flop / bf16 peak, weight bytes / HBM peak) + max(attention bytes / HBM peak, attention flop / bf16 peak)"},
        "stage_ms_per_step": stage_ms,
        "attention": {"us_per_layer": attn_s * 1e6, "GBps": (kv_bytes + qo_bytes) / attn_s / 1e9,
                      "hbm_frac": (kv_bytes + qo_bytes) / attn_s / 1e9 / PEAK_HBM_GBS,
                      "TFLOPs": attn_flops / attn_s / 1e12, "mfma_frac": attn_flops / attn_s / 1e12 / PEAK_BF16_TFLOPS,
                      "flop_per_byte": attn_flops / (kv_bytes + qo_bytes),
                      "bound": "hbm" if (kv_bytes + qo_bytes) / (PEAK_HBM_GBS * 1e9) >= attn_flops / (PEAK_BF16_TFLOPS * 1e12) else "mfma",
                      "frac_of_bound": attn_bound_s / attn_s},
        "gemm": {"TFLOPs": {k: v / (stage_ms[k] / L * 1e-3) / 1e12 for k, v in gemm_flops.items()},
                 "mfma_frac": {k: v / (stage_ms[k] / L * 1e-3) / 1e12 / PEAK_BF16_TFLOPS for k, v in gemm_flops.items()},
                 "aggregate_TFLOPs": sum(gemm_flops.values()) / gemm_s / 1e12,
                 "aggregate_mfma_frac": sum(gemm_flops.values()) / gemm_s / 1e12 / PEAK_BF16_TFLOPS,
                 "dominant_kernel": {"kernel": gu_kernel, "avg_launch_ms": gu_avg_ms, "launches": n,
                                     "flops_per_launch": gu_flops, "TFLOPs": gu_achieved,
                                     "mfma_frac": gu_achieved / PEAK_BF16_TFLOPS}},
    }
    if cpu_layers != 0:
        entry["cpu_baseline"] = cpu_baseline(name, w, sess, L if cpu_layers < 0 else min(cpu_layers, L))
    model.close()
    del sess, hidden, scores, esc
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    return entry


def run_alg1(n_questions=16, prompt=512, max_step_tokens=16, alg_steps=4, quantized_draft=False):
    """Algorithm 1 end to end on three synthetic roles (draft: 1.5B shape, or with quantized_draft the 8B shape with
    4-bit projection weights, the Q4-8B/8B/1.5B regime of Section 5.3; target: 8B shape; router: 1.5B shape with
    the linear head; random-init weights, a common vocabulary): reasoning steps per second of the whole loop
    (draft step token by token, router score, target step for the escalated sequences).  The separator is a
    token the random draft really emits and the threshold the median of a probe pass's scores, so steps end
    early for some sequences and both branches of the rule are taken."""
    from dataclasses import replace

    import numpy as np
    import torch

    import harness
    import paper_2512_05033_amd as A
    import workloads as W
    from paper_2512_05033_amd.arbitrage import Arbitrage, Role

    vocab = min(W.C2.model.vocab, W.C3.model.vocab)
    blocks_per_seq = (prompt + (alg_steps + 1) * max_step_tokens + 15) // 16 + 1
    n_blocks = n_questions * blocks_per_seq
    tables = np.random.default_rng(5).permutation(n_blocks).astype(np.int32).reshape(n_questions, blocks_per_seq)

    def role(name, shape, seed, lm, four_bit=False):
        m = replace(shape, vocab=vocab)
        weights = W.make_weights(m, seed, "cuda")
        if four_bit:
            weights = A.QuantizedWeights(weights)
        model = harness.make_model(m, weights, has_router_head=not lm)
        dims = (n_blocks, m.n_kv_heads, m.kv_block, m.head_dim)
        kv = A.KVCache([torch.zeros(dims, dtype=torch.bfloat16, device="cuda") for _ in range(m.n_layers)],
                       [torch.zeros(dims, dtype=torch.bfloat16, device="cuda") for _ in range(m.n_layers)])
        w_lm = W.normal_bf16(seed, "lm_head", (m.vocab, m.d_model), 0.02, "cuda") if lm else None
        return Role(name, model, kv, w_lm)

    draft = role("draft", W.C3.model, 11, True, four_bit=True) if quantized_draft else role("draft", W.C2.model, 11, True)
    roles = {"draft": draft, "target": role("target", W.C3.model, 12, True), "router": role("router", W.C2.model, 13, False)}
    questions = [[int(t) for t in W.uniform_ints(21, f"q{b}", prompt, vocab).numpy()] for b in range(n_questions)]

    def run(tau, sep, steps):
        for r in roles.values():
            r.fed = {}
        trace = []
        arb = Arbitrage(roles["draft"], roles["target"], roles["router"], tables, tau=tau, sep=sep, eos=-5,
                        max_step_tokens=max_step_tokens, trace=trace)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out, log = arb.run(questions, steps)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, out, log, trace

    _, _, log0, trace0 = run(1e9, -7, 1)                       # probe (also the warm-up)
    drafted = [e[4] for e in trace0 if e[0] == "step" and e[1] == "draft"]
    sep = drafted[0][min(5, len(drafted[0]) - 1)]
    tau = float(np.median([sc for b in log0 for sc, _ in log0[b]]))
    dt, out, log, trace = run(tau, sep, alg_steps)
    n_steps = sum(len(v) for v in log.values())
    n_esc = sum(e for v in log.values() for _, e in v)
    gen = sum(len(e[4]) for e in trace if e[0] == "step")
    for r in roles.values():
        r.model.close()
    return {"steps_per_s": n_steps / dt, "generated_tokens_per_s": gen / dt, "seconds": dt, "questions": n_questions,
            "prompt_tokens": prompt, "max_step_tokens": max_step_tokens, "alg1_steps": n_steps, "escalated": int(n_esc),
            "generated_tokens": gen, "mean_step_tokens": gen / max(1, sum(1 for e in trace if e[0] == "step")),
            "roles": ("draft 8B shape with 4-bit projection weights" if quantized_draft else "draft 1.5B shape") +
                     ", target 8B shape, router 1.5B shape + linear head; random-init, bf16"}


def run_few_token_forward(reps=20):
    """One drafting step's forward: the 1.5B shape, 16 sequences with one new token each against 2048 cached tokens
    (what every token position of Algorithm 1's draft loop costs).  Milliseconds per forward and, by the library's
    event hook, microseconds per layer and stage; the weights alone would take 2.62 GB / 8 TB/s = 0.33 ms."""
    from dataclasses import replace

    import torch

    import harness
    import paper_2512_05033_amd as A
    import workloads as W

    w = replace(W.C2, batch=16, step=("fixed", 1, 1), name="D1-draft1.5B-b16-p2048-s1")
    sess = harness.setup(w, "cuda")
    batch, model, m = sess.batch, sess.model, w.model
    hidden = torch.empty(batch.total_tokens, m.d_model, dtype=torch.bfloat16, device="cuda")
    scores = torch.empty(batch.batch, dtype=torch.float32, device="cuda")
    esc = torch.empty(batch.batch, dtype=torch.uint8, device="cuda")

    def step():
        A.arb_score_steps(model, sess.kv, sess.dbatch, batch.tau, ws=sess.ws, scores=scores, escalate=esc, hidden=hidden)

    for _ in range(5):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / reps * 1e3
    ids = {"qkv": A.ARB_STAGE_QKV, "attention": A.ARB_STAGE_ATTENTION, "oproj": A.ARB_STAGE_OPROJ,
           "gate_up": A.ARB_STAGE_GATE_UP, "down": A.ARB_STAGE_DOWN, "norm": A.ARB_STAGE_NORM,
           "rope_append": A.ARB_STAGE_ROPE_APPEND}
    stage_us = {}
    for sname in STAGES:
        t = A.StageTimer(model, ids[sname], 3 * m.n_layers)
        t.arm()
        for _ in range(3):
            step()
        torch.cuda.synchronize()
        dur = t.durations_ms(t.disarm())
        t.close()
        stage_us[sname] = round(sum(dur) / 3 / m.n_layers * 1e3, 2)
    model.close()
    weight_gb = m.n_layers * 2 * (m.qkv_rows * m.d_model + m.d_model * m.n_q_heads * m.head_dim + 3 * m.d_ffn * m.d_model) / 1e9
    return {"workload": w.name, "step_tokens": batch.total_tokens, "ms_per_forward": ms, "weights_GB": round(weight_gb, 3),
            "weights_TBps": round(weight_gb / ms, 3), "stage_us_per_layer": stage_us}


def run_w4_few_tokens(rows=16, reps=12):
    """The quantized-draft projections at a handful of tokens (Section 5.1's weight-quantized drafts, drafting token
    by token): each 4-bit projection of the 8B and 1.5B shapes at `rows` activation rows (gate/up also at 128), beside
    the bf16 kernel on the same shape; microseconds per launch by HIP events over launches that rotate through four copies of the
    weights (so that they come from memory), and the packed-weight bytes per second that is."""
    import torch

    import paper_2512_05033_amd as A

    g = torch.Generator(device="cuda").manual_seed(7)

    def per_launch_us(fn):
        for i in range(4):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    out = []
    for label, n, k, epi in [("8B gate/up", 14336, 4096, A.ARB_EPI_SWIGLU_BF16), ("8B down", 4096, 14336, A.ARB_EPI_STORE_F32),
                             ("8B QKV", 6144, 4096, A.ARB_EPI_STORE_BF16), ("1.5B gate/up", 8960, 1536, A.ARB_EPI_SWIGLU_BF16),
                             ("1.5B down", 1536, 8960, A.ARB_EPI_STORE_F32)]:
        w_rows = 2 * n if epi == A.ARB_EPI_SWIGLU_BF16 else n
        dense = [(torch.randn(w_rows, k, device="cuda", generator=g) * 0.05).bfloat16() for _ in range(4)]
        packed = [A.arb_w4_quantize(w) for w in dense]
        for m in ([rows, 128] if "gate/up" in label else [rows]):       # 128 rows: the tile kernel (one tile row)
            x = torch.randn(m, k, device="cuda", generator=g).bfloat16()
            us4 = per_launch_us(lambda i: A.arb_stage_gemm_w4(x, *packed[i % 4], epi))
            us16 = per_launch_us(lambda i: A.arb_stage_gemm(x, dense[i % 4], epi))
            out.append({"projection": label, "rows": m, "weight_rows": w_rows, "K": k, "w4_us": round(us4, 2),
                        "bf16_us": round(us16, 2), "packed_weight_TBps": round(w_rows * k / 2 / us4 / 1e6, 3)})
        del dense, packed
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C2", help="the workload of the headline value")
    ap.add_argument("--configs", default="C2,C3,C4,C5", help="workloads reported in per_config (comma separated; '' = only the headline)")
    ap.add_argument("--cpu-layers", type=int, default=-1, help="layers of the oracle sample (-1 = all, 0 = skip the CPU baseline)")
    ap.add_argument("--breakdown", action="store_true", help="kept for compatibility: stage times are always reported")
    ap.add_argument("--stage-reps", type=int, default=3, help="extra passes per stage for the per-stage times (0: none, "
                    "for hardware-counter runs; per_config then holds the step times only)")
    ap.add_argument("--alg1", type=int, default=1, help="1: also time Algorithm 1 end to end on three synthetic roles (field alg1)")
    ap.add_argument("--w4", type=int, default=1, help="1: also time one few-token forward (field few_token_forward) and the 4-bit projections at 16 rows beside the bf16 ones (field w4_few_tokens)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="before the warm-up, run one plain device copy of this many MiB (a kernel of known traffic "
                         "that hardware-counter runs are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU (sequences are independent, so a batch would shard by "
                 "sequence across GPUs with no communication on the path); run with --gpus 1")

    import torch

    import paper_2512_05033_amd as A

    A.load_library()
    torch.cuda.set_device(0)
    names = [args.workload] + [c for c in args.configs.split(",") if c and c != args.workload]
    per_config = []
    for i, name in enumerate(names):
        per_config.append(run_config(name, args.steps, args.warmup, args.cpu_layers,
                                     args.copy_probe_mib if i == 0 else 0, args.stage_reps))
        print(f"bench: {name} done: {per_config[-1]['ms_per_step']:.3f} ms per step", file=sys.stderr, flush=True)
    per_config.sort(key=lambda e: e["workload"])
    head = next(e for e in per_config if e["workload"].startswith(args.workload))
    dom = head["gemm"]["dominant_kernel"]
    # HBM-side bytes per launch of that kernel from the FETCH_SIZE / WRITE_SIZE counter runs
    # (profiles/score_steps_C2_hbm_traffic.txt); only valid for the kernel source they were taken with
    traffic = None
    with open(os.path.join(os.path.dirname(os.path.abspath(A.__file__)), "csrc", "gemm.hip"), "rb") as f:
        if args.workload == "C2" and hashlib.sha256(f.read()).hexdigest() == COUNTED_GEMM_SHA256:
            traffic = COUNTED_GATE_UP_BYTES
    out = {
        "metric": "scored step-tokens/sec on 1 MI355X", "value": head["step_tokens_per_s"], "unit": "scored step-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": head["workload"], "layers": head["layers"], "d_model": head["d_model"], "batch": head["batch"],
                   "prefix_tokens": head["prefix_tokens"], "step_tokens": head["step_tokens"], "kv": head["kv"]},
        "roofline": {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom["TFLOPs"],
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": dom["mfma_frac"], "traffic": traffic,
                     "avg_launch_ms": dom["avg_launch_ms"], "launches": dom["launches"],
                     "flops_per_launch": dom["flops_per_launch"]},
        "per_config": per_config,
    }
    if args.stage_reps > 0:
        out["attention_hbm_frac"] = {e["workload"].split("-")[0]: round(e["attention"]["hbm_frac"], 4) for e in per_config}
        out["gemm_mfma_frac"] = {e["workload"].split("-")[0]: round(e["gemm"]["aggregate_mfma_frac"], 4) for e in per_config}
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    if args.alg1 and args.stage_reps > 0:
        out["alg1"] = run_alg1()
        print(f"bench: Algorithm 1 done: {out['alg1']['steps_per_s']:.1f} steps per second", file=sys.stderr, flush=True)
        torch.cuda.empty_cache()
        out["alg1_q4_draft"] = run_alg1(quantized_draft=True)
        print(f"bench: Algorithm 1 with the 4-bit draft done: {out['alg1_q4_draft']['steps_per_s']:.1f} steps per second",
              file=sys.stderr, flush=True)
    if args.w4 and args.stage_reps > 0:
        out["few_token_forward"] = run_few_token_forward()
        print(f"bench: few-token forward done: {out['few_token_forward']['ms_per_forward']:.3f} ms", file=sys.stderr, flush=True)
        out["w4_few_tokens"] = run_w4_few_tokens()
        print("bench: 4-bit projections at 16 rows done", file=sys.stderr, flush=True)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
