"""Benchmark of the step-scoring hot path on one MI355X.

A step = one arb_score_steps call (embedding, L transformer layers of
append-attention + projections, final norm, pooled router head, threshold) over
one batch of the 1.5B-router-shaped workload (16 sequences, 2048-token cached
prefix, 64-token drafted step), inputs resident in HBM.  Prints one JSON line.
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
COUNTED_GATE_UP_BYTES = 75791902 + 16777216
COUNTED_GEMM_SHA256 = "b92d31b84caa34adf6078b6498e96b8c33086020f1e92ebbd1713c867cefe0f5"


def cpu_baseline(w, sess, layers: int):
    """The CPU oracle, as it stands, on a bounded sample: the full batch through
    the first `layers` layers plus final norm and head; scaled to full depth."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info

    import workloads as W
    from helpers import oracle_model, oracle_params
    from oracle import arb_oracle as O

    sub = W.scaled(w, n_layers=layers)
    wt = sess.weights
    cpu = lambda t: t.cpu()
    weights = W.Weights(cpu(wt.embed), [cpu(t) for t in wt.wqkv[:layers]], [cpu(t) for t in wt.wo[:layers]],
                        [cpu(t) for t in wt.wgu[:layers]], [cpu(t) for t in wt.wd[:layers]],
                        [cpu(t) for t in wt.g_attn[:layers]], [cpu(t) for t in wt.g_mlp[:layers]], cpu(wt.g_final),
                        cpu(wt.w_head), wt.b_head)
    m, p = oracle_model(sub.model), oracle_params(weights)
    batch = sess.batch
    kp = [W.bf16_bits(sess.kv.k_pools[l]).copy() for l in range(layers)]
    vp = [W.bf16_bits(sess.kv.v_pools[l]).copy() for l in range(layers)]
    t0 = time.perf_counter()
    O.score_steps(m, p, kp, vp, batch.token_ids, batch.prefix_lens, batch.cu_step_lens, batch.block_tables, batch.tau)
    dt = time.perf_counter() - t0
    threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    full = dt * w.model.n_layers / layers
    return {"value": batch.total_tokens / full, "unit": "scored step-tokens/s", "cores": int(threads),
            "kind": "oracle",
            "sample": f"full batch ({batch.batch} seq, {batch.total_tokens} step tokens) through the first {layers} of "
                      f"{w.model.n_layers} layers + head in {dt:.1f} s; value = tokens / (time x {w.model.n_layers}/{layers})"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--cpu-layers", type=int, default=-1, help="layers of the oracle sample (-1 = all, 0 = skip the CPU baseline)")
    ap.add_argument("--breakdown", action="store_true", help="also time each stage (extra passes, not in the timed region)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="before the warm-up, run one plain device copy of this many MiB (a kernel of known traffic "
                         "that hardware-counter runs are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU (sequences are independent, so a batch would shard by "
                 "sequence across GPUs with no communication on the path); run with --gpus 1")

    import torch

    import paper_2512_05033_amd as A
    import workloads as W
    import harness

    A.load_library()
    torch.cuda.set_device(0)
    w = W.ALL[args.workload]
    sess = harness.setup(w, "cuda")
    batch, model = sess.batch, sess.model
    T, L = batch.total_tokens, w.model.n_layers
    head = w.model.has_router_head
    scores = torch.empty(batch.batch, dtype=torch.float32, device="cuda") if head else None
    esc = torch.empty(batch.batch, dtype=torch.uint8, device="cuda") if head else None
    hidden = torch.empty(T, w.model.d_model, dtype=torch.bfloat16, device="cuda")

    def step():
        A.arb_score_steps(model, sess.kv, sess.dbatch, batch.tau, ws=sess.ws, scores=scores, escalate=esc,
                          hidden=hidden)

    if args.copy_probe_mib > 0:
        src = torch.arange(args.copy_probe_mib << 18, dtype=torch.float32, device="cuda")   # 4 bytes each
        torch.empty_like(src).copy_(src)
        del src
    for _ in range(args.warmup):
        step()
    # The dominant kernel is bracketed by HIP events inside the library, on the stream it runs on,
    # during the timed steps: the gate/up projection with the SwiGLU epilogue, or, where that
    # projection is launched as two kernels, the 256x256-tile kernel that does most of its columns.
    F, d = w.model.d_ffn, w.model.d_model
    large_cols = A.arb_gemm_large_tile_columns(T, F, d, A.ARB_EPI_SWIGLU_BF16)
    if large_cols > 0:
        gu_stage, gu_features = A.ARB_STAGE_GATE_UP_LARGE, large_cols * 128
        gu_kernel = f"gemm256_kernel<SWIGLU, K-blocked weights> (gate/up projection, features [0, {gu_features}) of {F} in 256x256 tiles)"
    else:
        gu_stage, gu_features = A.ARB_STAGE_GATE_UP, F
        gu_kernel = "gemm_kernel<SWIGLU> (gate/up projection, 128x128 tiles)"
    timer = A.StageTimer(model, gu_stage, args.steps * L)
    timer.arm()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    n = timer.disarm()
    gu_ms = timer.durations_ms(n)
    timer.close()
    ms_per_step = dt / args.steps * 1e3
    gu_avg_ms = sum(gu_ms) / len(gu_ms)
    gu_flops = 2.0 * T * (2 * gu_features) * d                            # per launch of that kernel
    achieved = gu_flops / (gu_avg_ms * 1e-3) / 1e12
    # HBM-side bytes per launch of that kernel from the FETCH_SIZE / WRITE_SIZE counter runs
    # (profiles/score_steps_C2_hbm_traffic.txt); only valid for the kernel source they were taken with
    traffic = None
    with open(os.path.join(os.path.dirname(os.path.abspath(A.__file__)), "csrc", "gemm.hip"), "rb") as f:
        if args.workload == "C2" and hashlib.sha256(f.read()).hexdigest() == COUNTED_GEMM_SHA256:
            traffic = COUNTED_GATE_UP_BYTES

    out = {
        "metric": "scored step-tokens/sec on 1 MI355X", "value": T / (ms_per_step * 1e-3), "unit": "scored step-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "layers": L, "d_model": w.model.d_model, "batch": batch.batch,
                   "prefix_tokens": int(batch.prefix_lens.sum()), "step_tokens": T, "kv": f"paged-16 {w.tables}"},
        "roofline": {"bound": "mfma", "kernel": gu_kernel, "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "avg_launch_ms": gu_avg_ms, "launches": n, "flops_per_launch": gu_flops},
    }

    if args.breakdown:
        stages = {"qkv": A.ARB_STAGE_QKV, "attention": A.ARB_STAGE_ATTENTION, "oproj": A.ARB_STAGE_OPROJ,
                  "gate_up": A.ARB_STAGE_GATE_UP, "down": A.ARB_STAGE_DOWN, "norm": A.ARB_STAGE_NORM,
                  "rope_append": A.ARB_STAGE_ROPE_APPEND}
        bd = {}
        for name, sid in stages.items():
            t = A.StageTimer(model, sid, 3 * L)
            t.arm()
            for _ in range(3):
                step()
            torch.cuda.synchronize()
            d = t.durations_ms(t.disarm())
            t.close()
            bd[name] = sum(d) / 3
        m = w.model
        kv_bytes = float(((batch.prefix_lens + batch.step_lens) * 2 * m.n_kv_heads * m.head_dim * 2).sum())
        attn_flops = float(4 * m.n_q_heads * m.head_dim * (batch.step_lens * batch.prefix_lens + batch.step_lens * (batch.step_lens + 1) / 2).sum())
        qo_bytes = 2.0 * T * m.n_q_heads * m.head_dim * 2
        out["stage_ms_per_step"] = bd
        out["attention"] = {"ms_per_layer": bd["attention"] / L, "GBps": (kv_bytes + qo_bytes) / (bd["attention"] / L * 1e-3) / 1e9,
                            "hbm_frac": (kv_bytes + qo_bytes) / (bd["attention"] / L * 1e-3) / 1e9 / PEAK_HBM_GBS,
                            "TFLOPs": attn_flops / (bd["attention"] / L * 1e-3) / 1e12}
        gemm_flops = {"qkv": 2.0 * T * m.qkv_rows * m.d_model, "oproj": 2.0 * T * m.d_model * m.n_q_heads * m.head_dim,
                      "gate_up": 2.0 * T * 2 * m.d_ffn * m.d_model, "down": 2.0 * T * m.d_model * m.d_ffn}
        out["gemm_TFLOPs"] = {k: v / (bd[k] / L * 1e-3) / 1e12 for k, v in gemm_flops.items()}

    if args.cpu_layers < 0:
        args.cpu_layers = L
    if args.cpu_layers > 0:
        out["cpu_baseline"] = cpu_baseline(w, sess, min(args.cpu_layers, L))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
