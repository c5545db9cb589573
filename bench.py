#!/usr/bin/env python3
"""Benchmark of the CritiPrefill prefill-attention path on one MI355X.

A "step" is one pass of the whole hot path over one synthetic layer:
critiprefill_estimate -> critiprefill_select -> critiprefill_sparse_attn, inputs resident in HBM.
Default workload: the Llama3-8B-shaped layer at 128K tokens (32 query / 8 KV heads, d=128, bf16,
segment 512, block 64, budget 2048 tokens + diagonal + 1 local block).

Prints ONE JSON line: the per-layer latency (the headline metric), the speedup over the library's own
dense causal kernel, the roofline of the dominant kernel (block-sparse attention, bf16 MFMA-bound) and
the CPU checker timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published


def read_traffic(workload: str):
    """HBM bytes per sparse_attn launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE), if a
    summary for this workload has been committed under profiles/."""
    path = os.path.join(ROOT, "profiles", f"sparse_attn_{workload}_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3_llama3_8b_128k")
    ap.add_argument("--dense-steps", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy (a known-size kernel to scale rocprofv3 FETCH_SIZE/WRITE_SIZE by)")
    ap.add_argument("--cpu-heads", type=int, default=8, help="query heads the CPU checker estimates, selects and attends")
    ap.add_argument("--cpu-segments", type=int, default=1280, help="(head, segment) pairs the CPU checker attends, over all sampled heads")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2409_12490_amd import binding as B
    from paper_2409_12490_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.load()                                     # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    t0 = time.time()
    q_h, k_h, v_h = synth.make_qkv(w, threads=min(16, os.cpu_count() or 8))
    gen_s = time.time() - t0
    q, k, v = q_h.to(dev), k_h.to(dev), v_h.to(dev)
    out = torch.empty_like(q)
    p = B.make_params(q, k, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks, out=out)
    S = B.alloc_scores(p, dev)
    ws = B.alloc_workspace(p, dev)
    idx, cnt = B.alloc_lists(p, dev)

    def step(events=None):
        if events is not None:
            events[0].record()
        B.critiprefill_estimate(p, q, k, None, S, ws)
        if events is not None:
            events[1].record()
        B.critiprefill_select(p, S, idx, cnt)
        if events is not None:
            events[2].record()
        B.critiprefill_sparse_attn(p, q, k, v, idx, cnt, out, None)
        if events is not None:
            events[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # HIP events on the stream the kernels are launched on (torch's current stream)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    est_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    sel_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
    att_ms = float(np.mean([e[2].elapsed_time(e[3]) for e in evs]))
    layer_ms = np.array([e[0].elapsed_time(e[3]) for e in evs])      # per step, HIP events on the launch stream

    # algorithmic work of the sparse attention: 4*d flop per visited (query, key <= query) pair
    d, s, b, r, n = w.head_dim, w.segment_size, w.block_size, w.blocks_per_segment, w.seq_len
    assert n % s == 0
    cnt_sum = int(cnt.to(torch.int64).sum().item())
    rows = w.batch * w.n_q_heads * w.n_segments
    pairs = (cnt_sum - rows * r) * b * s + rows * (s * (s + 1) // 2)
    sparse_flop = 4.0 * d * pairs
    dense_flop = 4.0 * d * w.batch * w.n_q_heads * (n * (n + 1) // 2)
    est_bytes = (w.n_q_heads + w.n_kv_heads) * w.batch * n * d * q.element_size() + S.numel() * 4

    # the library's own dense causal kernel on the same tensors
    dense_out = torch.empty_like(q)
    B.critiprefill_dense_causal_attn(p, q, k, v, dense_out, None)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.dense_steps):
        B.critiprefill_dense_causal_attn(p, q, k, v, dense_out, None)
    e1.record()
    torch.cuda.synchronize()
    dense_ms = e0.elapsed_time(e1) / args.dense_steps
    sparse_vs_dense_err = float((out.float() - dense_out.float()).abs().max().item())

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    achieved = sparse_flop / (att_ms * 1e-3) / 1e12
    result = {
        "metric": "prefill_attn_latency_per_layer_128k" if n == 131072 else "prefill_attn_latency_per_layer",
        "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": d, "seq_len": n, "segment": s, "block": b, "budget_blocks": w.budget_blocks,
                   "local_blocks": w.local_blocks},
        "layer_ms_p10_p50_p90": [round(float(np.percentile(layer_ms, q)), 4) for q in (10, 50, 90)],
        "breakdown_ms": {"estimate": round(est_ms, 4), "select": round(sel_ms, 4), "sparse_attn": round(att_ms, 4),
                         "dense_causal_attn": round(dense_ms, 3)},
        "speedup_vs_dense": round(dense_ms / ms_per_step, 3),
        "sparse_attn_speedup_vs_dense_kernel": round(dense_ms / att_ms, 3),
        "effective_tflops": round(achieved, 1),
        "dense_tflops": round(dense_flop / (dense_ms * 1e-3) / 1e12, 1),
        "mfma_util": round(achieved / PEAK_BF16_TFLOPS, 4),
        "estimate_gbps": round(est_bytes / (est_ms * 1e-3) / 1e9, 1),
        "estimate_hbm_frac": round(est_bytes / (est_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        "sparse_vs_dense_max_abs": round(sparse_vs_dense_err, 4),
        "input_gen_s": round(gen_s, 1),
        "roofline": {"kernel": "attn_bf16_kernel<sparse>", "bound": "mfma", "achieved": round(achieved, 1),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": read_traffic(w.name), "flop_per_launch": sparse_flop,
                     "avg_launch_ms": round(att_ms, 4)},
    }

    if not args.no_cpu_baseline:
        # the CPU checker as it stands, on a bounded sample (10-30 s of CPU work): Algorithm 1 + top-k for a few
        # query heads, then the pruned attention of some of their segments; scaled linearly to one whole layer.
        from oracle import critiprefill_oracle as O
        nh = max(1, min(args.cpu_heads, w.n_q_heads))
        heads = sorted(set(int(round(i * (w.n_q_heads - 1) / max(nh - 1, 1))) for i in range(nh)))
        G = w.n_q_heads // w.n_kv_heads
        t0 = time.perf_counter()
        lists = {}
        for h in heads:
            qf = synth.to_f64(q_h[:, h:h + 1]); kf = synth.to_f64(k_h[:, h // G:h // G + 1])
            S_o = O.estimate(qf, kf, s, b)
            lists[h] = O.select(O.scores_in_decision_precision(S_o), s, b, w.budget_blocks, w.local_blocks)
        t_est = time.perf_counter() - t0
        rng = np.random.default_rng(0)
        per_head = max(1, args.cpu_segments // len(heads))
        segs = sorted(int(x) for x in rng.choice(np.arange(w.n_segments // 4, w.n_segments), size=min(per_head, w.n_segments - w.n_segments // 4), replace=False))
        t0 = time.perf_counter()
        worst = 0.0
        n_done = 0
        for h in heads:
            qf = synth.to_f64(q_h[:, h:h + 1]); kf = synth.to_f64(k_h[:, h // G:h // G + 1])
            vf = synth.to_f64(v_h[:, h // G:h // G + 1])
            idx_o, cnt_o = lists[h]
            todo = [(0, 0, j) for j in segs]
            o_ref, _ = O.sparse_attention(qf, kf, vf, idx_o, cnt_o, s, b, segments=todo)
            n_done += len(todo)
            # parity on the sampled segments, with the GPU's own list when it equals the checker's
            idx_g = idx[0, h].cpu().numpy(); cnt_g = cnt[0, h].cpu().numpy()
            for (_, _, j) in todo:
                if np.array_equal(idx_g[j], idx_o[0, 0, j]):
                    got = out[0, h, j * s:(j + 1) * s].float().cpu().numpy()
                    worst = max(worst, float(np.abs(got - o_ref[0, 0, j * s:(j + 1) * s]).max()))
        t_att = time.perf_counter() - t0
        cpu_layer_ms = (t_est / len(heads) * w.n_q_heads * w.batch + t_att / n_done * rows) * 1e3
        result["cpu_baseline"] = {
            "value": round(cpu_layer_ms, 1), "unit": "ms", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
            "kind": "oracle",
            "sample": f"fp64 numpy checker: estimate+select of {len(heads)} of {w.n_q_heads} heads ({t_est:.1f} s) and pruned "
                      f"attention of {n_done} of {rows} (head, segment) pairs ({t_att:.1f} s), scaled linearly to one layer",
            "sampled_output_max_abs_err": round(worst, 5),
        }
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
