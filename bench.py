#!/usr/bin/env python3
"""Benchmark of the CritiPrefill prefill-attention path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input, inputs resident in HBM:
critiprefill_estimate -> critiprefill_select -> critiprefill_sparse_attn for every layer of the workload.

Default workload: the Llama3-8B-shaped layer at 128K tokens (32 query / 8 KV heads, d=128, bf16, segment 512,
block 64, budget 2048 tokens + diagonal + 1 local block), the configuration the headline metric is quoted on.
It prints ONE JSON line: the per-layer latency, the speedup over the library's own dense causal kernel, the
roofline of the dominant kernel (block-sparse attention, bf16 MFMA-bound) and the CPU checker timed on a
bounded sample of the same workload.

``--workload c5_llama3_8b_64k_x4`` runs the 4-layer stack (batch 2, 64K tokens, segment 256, block 32, layer
fusion S = 0.5 S + 0.5 S') and prints one JSON line per token budget (512 / 1024 / 4096): per-layer and total
latency, speedup over the dense kernel, and the output error against the dense kernel and against the checker.
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
INFINITY_CACHE_BYTES = 256 << 20


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


def pct(xs, np):
    """[p10, p50, p90] of a list of milliseconds."""
    return [round(float(np.percentile(xs, q)), 4) for q in (10, 50, 90)]


def sparse_pairs(w, cnt_sum: int) -> int:
    """Visited (query, key <= query) pairs of a launch: listed past blocks in full, the diagonal token-exact."""
    s, b, r = w.segment_size, w.block_size, w.blocks_per_segment
    rows = w.batch * w.n_q_heads * w.n_segments
    return (cnt_sum - rows * r) * b * s + rows * (s * (s + 1) // 2)


def cpu_threads() -> str:
    n = os.environ.get("OMP_NUM_THREADS", str(os.cpu_count() or 1))
    return (f"numpy checker: python loops on one thread, matrix products on up to {n} BLAS threads; "
            "cores = CPU time / wall time of the sample")


def cpu_baseline_layer(O, synth, np, w, q_h, k_h, v_h, idx, cnt, out, n_heads, n_segments, prev=None, alpha=1.0):
    """The CPU checker as it stands on a bounded sample of one layer: Algorithm 1 + top-k for a few (batch, head)
    pairs, the pruned attention of some of their segments; scaled linearly to the whole layer.  Also compares the
    library's output on those segments (only where its list equals the checker's; both counts are reported).
    Returns (record, checker scores per sampled (batch, head))."""
    s, b = w.segment_size, w.block_size
    G = w.n_q_heads // w.n_kv_heads
    rows = w.batch * w.n_q_heads * w.n_segments
    nh = max(1, min(n_heads, w.batch * w.n_q_heads))
    flat = sorted(set(int(round(i * (w.batch * w.n_q_heads - 1) / max(nh - 1, 1))) for i in range(nh)))
    heads = [(x // w.n_q_heads, x % w.n_q_heads) for x in flat]
    t0 = time.perf_counter()
    c0 = time.process_time()
    lists, scores = {}, {}
    for (bb, h) in heads:
        qf = synth.to_f64(q_h[bb:bb + 1, h:h + 1]); kf = synth.to_f64(k_h[bb:bb + 1, h // G:h // G + 1])
        S_o = O.estimate(qf, kf, s, b, prev_scores=None if prev is None else prev[(bb, h)], alpha=alpha)
        scores[(bb, h)] = S_o
        lists[(bb, h)] = O.select(O.scores_in_decision_precision(S_o), s, b, w.budget_blocks, w.local_blocks)
    t_est = time.perf_counter() - t0
    rng = np.random.default_rng(0)
    per_head = max(1, n_segments // len(heads))
    lo = w.n_segments // 4
    segs = sorted(int(x) for x in rng.choice(np.arange(lo, w.n_segments), size=min(per_head, w.n_segments - lo), replace=False))
    t0 = time.perf_counter()
    worst, n_done, n_same = 0.0, 0, 0
    for (bb, h) in heads:
        qf = synth.to_f64(q_h[bb:bb + 1, h:h + 1]); kf = synth.to_f64(k_h[bb:bb + 1, h // G:h // G + 1])
        vf = synth.to_f64(v_h[bb:bb + 1, h // G:h // G + 1])
        idx_o, cnt_o = lists[(bb, h)]
        todo = [(0, 0, j) for j in segs]
        o_ref, _ = O.sparse_attention(qf, kf, vf, idx_o, cnt_o, s, b, segments=todo)
        n_done += len(todo)
        idx_g = idx[bb, h].cpu().numpy()
        for (_, _, j) in todo:
            if np.array_equal(idx_g[j], idx_o[0, 0, j]):
                n_same += 1
                got = out[bb, h, j * s:(j + 1) * s].float().cpu().numpy()
                worst = max(worst, float(np.abs(got - o_ref[0, 0, j * s:(j + 1) * s]).max()))
    t_att = time.perf_counter() - t0
    cores = round((time.process_time() - c0) / max(t_est + t_att, 1e-9), 1)
    cpu_layer_ms = (t_est / len(heads) * w.n_q_heads * w.batch + t_att / n_done * rows) * 1e3
    rec = {
        "value": round(cpu_layer_ms, 1), "unit": "ms", "cores": cores, "kind": "oracle", "threads": cpu_threads(),
        "sample": f"fp64 numpy checker: estimate+select of {len(heads)} of {w.batch * w.n_q_heads} (batch, head) pairs ({t_est:.1f} s) "
                  f"and pruned attention of {n_done} of {rows} (head, segment) pairs ({t_att:.1f} s), scaled linearly to one layer",
        "sampled_segments_compared": n_same, "sampled_segments_total": n_done,
        "sampled_output_max_abs_err": round(worst, 5) if n_same else None,
    }
    if n_same == 0:
        rec["warning"] = "no sampled segment had a list identical to the checker's: output error not measured"
    return rec, scores


def run_single_layer(args, np, torch, B, synth, w, dev):
    t0 = time.time()
    q_h, k_h, v_h = synth.make_qkv(w, threads=min(16, os.cpu_count() or 8))
    gen_s = time.time() - t0
    # rotate over several copies of the inputs when one copy would (nearly) fit the Infinity Cache, so that the
    # memory-bound estimate step reads HBM as it would in a model where other layers run in between
    in_bytes = (q_h.numel() + k_h.numel() + v_h.numel()) * q_h.element_size()
    n_rot = args.rotate if args.rotate > 0 else (4 if in_bytes < 2 * INFINITY_CACHE_BYTES else 1)
    bufs = [(q_h.to(dev), k_h.to(dev), v_h.to(dev)) for _ in range(n_rot)]
    q, k, v = bufs[0]
    out = torch.empty_like(q)
    p = B.make_params(q, k, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks, out=out)
    S = B.alloc_scores(p, dev)
    ws = B.alloc_workspace(p, dev)
    idx, cnt = B.alloc_lists(p, dev)

    def step(i, events=None):
        qi, ki, vi = bufs[i % n_rot]
        if events is not None:
            events[0].record()
        B.critiprefill_estimate(p, qi, ki, None, S, ws)
        if events is not None:
            events[1].record()
        B.critiprefill_select(p, S, idx, cnt)
        if events is not None:
            events[2].record()
        B.critiprefill_sparse_attn(p, qi, ki, vi, idx, cnt, out, None)
        if events is not None:
            events[3].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # HIP events on the stream the kernels are launched on (torch's current stream)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    est = [e[0].elapsed_time(e[1]) for e in evs]
    sel = [e[1].elapsed_time(e[2]) for e in evs]
    att = [e[2].elapsed_time(e[3]) for e in evs]
    layer_ms = [e[0].elapsed_time(e[3]) for e in evs]
    est_ms, sel_ms, att_ms = float(np.mean(est)), float(np.mean(sel)), float(np.mean(att))
    if (args.steps - 1) % n_rot != 0:            # leave the outputs of copy 0 behind for the checks below
        step(0)
        torch.cuda.synchronize()

    d, n = w.head_dim, w.seq_len
    sparse_flop = 4.0 * d * sparse_pairs(w, int(cnt.to(torch.int64).sum().item()))
    dense_flop = 4.0 * d * w.batch * w.n_q_heads * (n * (n + 1) // 2)
    est_bytes = (w.n_q_heads + w.n_kv_heads) * w.batch * n * d * q.element_size() + S.numel() * 4

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
                   "head_dim": d, "seq_len": n, "segment": w.segment_size, "block": w.block_size,
                   "budget_blocks": w.budget_blocks, "local_blocks": w.local_blocks, "input_copies_rotated": n_rot},
        "layer_ms_p10_p50_p90": pct(layer_ms, np),
        "breakdown_ms": {"estimate": round(est_ms, 4), "select": round(sel_ms, 4), "sparse_attn": round(att_ms, 4),
                         "dense_causal_attn": round(dense_ms, 3)},
        "breakdown_ms_p10_p50_p90": {"estimate": pct(est, np), "select": pct(sel, np), "sparse_attn": pct(att, np)},
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
        from oracle import critiprefill_oracle as O
        result["cpu_baseline"], _ = cpu_baseline_layer(O, synth, np, w, q_h, k_h, v_h, idx, cnt, out,
                                                       args.cpu_heads, args.cpu_segments)
    print(json.dumps(result), flush=True)


def run_stack(args, np, torch, B, synth, w, dev):
    """The multi-layer workload: every layer has its own Q/K/V, layer l's criticality scores are fused with the
    scores layer l-1 returned (Algorithm 1, last line); one JSON line per token budget."""
    t0 = time.time()
    host = [synth.make_qkv(w, layer=l, threads=min(16, os.cpu_count() or 8)) for l in range(w.layers)]
    gen_s = time.time() - t0
    layers = [(q.to(dev), k.to(dev), v.to(dev)) for (q, k, v) in host]
    q0, k0, _ = layers[0]
    out = [torch.empty_like(q0) for _ in range(w.layers)]
    dense_out = torch.empty_like(q0)
    d, n = w.head_dim, w.seq_len
    budgets = [int(x) for x in args.budgets.split(",")]
    p0 = B.make_params(q0, k0, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks, out=out[0], alpha=w.alpha)
    S = B.alloc_scores(p0, dev)
    ws = B.alloc_workspace(p0, dev)

    # the library's dense kernel on every layer: the speed baseline and the reference of the output error
    dense_ms, dense_keep = [], []
    for l, (q, k, v) in enumerate(layers):
        B.critiprefill_dense_causal_attn(p0, q, k, v, dense_out, None)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.dense_steps):
            B.critiprefill_dense_causal_attn(p0, q, k, v, dense_out, None)
        e1.record()
        torch.cuda.synchronize()
        dense_ms.append(e0.elapsed_time(e1) / args.dense_steps)
        dense_keep.append(dense_out.clone())
    dense_flop = 4.0 * d * w.batch * w.n_q_heads * (n * (n + 1) // 2)

    for budget_tokens in budgets:
        wb = w.replace(budget_blocks=budget_tokens // w.block_size)
        p = B.make_params(q0, k0, wb.segment_size, wb.block_size, wb.budget_blocks, wb.local_blocks, out=out[0], alpha=w.alpha)
        lists = [B.alloc_lists(p, dev) for _ in range(w.layers)]

        def step(events=None):
            for l, (q, k, v) in enumerate(layers):
                idx, cnt = lists[l]
                if events is not None:
                    events[l][0].record()
                B.critiprefill_estimate(p, q, k, S if l > 0 else None, S, ws)     # in place: S' is overwritten by S
                if events is not None:
                    events[l][1].record()
                B.critiprefill_select(p, S, idx, cnt)
                if events is not None:
                    events[l][2].record()
                B.critiprefill_sparse_attn(p, q, k, v, idx, cnt, out[l], None)
                if events is not None:
                    events[l][3].record()

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        evs = [[[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(w.layers)] for _ in range(args.steps)]
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(evs[i])
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
        per_layer = []
        for l in range(w.layers):
            est = [e[l][0].elapsed_time(e[l][1]) for e in evs]
            sel = [e[l][1].elapsed_time(e[l][2]) for e in evs]
            att = [e[l][2].elapsed_time(e[l][3]) for e in evs]
            tot = [e[l][0].elapsed_time(e[l][3]) for e in evs]
            diff = out[l].float() - dense_keep[l].float()
            per_layer.append({
                "layer": l, "ms": round(float(np.mean(tot)), 4), "ms_p10_p50_p90": pct(tot, np),
                "estimate_ms": round(float(np.mean(est)), 4), "select_ms": round(float(np.mean(sel)), 4),
                "sparse_attn_ms": round(float(np.mean(att)), 4), "dense_causal_attn_ms": round(dense_ms[l], 3),
                "speedup_vs_dense": round(dense_ms[l] / float(np.mean(tot)), 3),
                "vs_dense_max_abs": round(float(diff.abs().max().item()), 4),
                "vs_dense_rel_l2": round(float((diff.norm() / dense_keep[l].float().norm()).item()), 4),
            })
            del diff
        att_ms = float(np.mean([x["sparse_attn_ms"] for x in per_layer]))
        cnt_sum = sum(int(c.to(torch.int64).sum().item()) for (_, c) in lists) / w.layers
        sparse_flop = 4.0 * d * sparse_pairs(wb, int(cnt_sum))
        achieved = sparse_flop / (att_ms * 1e-3) / 1e12
        result = {
            "metric": f"prefill_attn_latency_{w.layers}_layers", "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": False,
            "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
            "config": {"workload": w.name, "layers": w.layers, "fusion_alpha": w.alpha, "batch": w.batch,
                       "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "head_dim": d, "seq_len": n,
                       "segment": w.segment_size, "block": w.block_size, "budget_tokens": budget_tokens,
                       "budget_blocks": wb.budget_blocks, "local_blocks": wb.local_blocks},
            "per_layer": per_layer,
            "dense_total_ms": round(sum(dense_ms), 3),
            "speedup_vs_dense": round(sum(dense_ms) / ms_per_step, 3),
            "vs_dense_max_abs": max(x["vs_dense_max_abs"] for x in per_layer),
            "vs_dense_rel_l2": round(float(np.mean([x["vs_dense_rel_l2"] for x in per_layer])), 4),
            "effective_tflops": round(achieved, 1),
            "dense_tflops": round(dense_flop / (float(np.mean(dense_ms)) * 1e-3) / 1e12, 1),
            "input_gen_s": round(gen_s, 1),
            "roofline": {"kernel": "attn_bf16_kernel<sparse, 32-token blocks>", "bound": "mfma", "achieved": round(achieved, 1),
                         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                         "traffic": read_traffic(f"{w.name}_b{budget_tokens}"), "flop_per_launch": sparse_flop,
                         "avg_launch_ms": round(att_ms, 4)},
        }
        if not args.no_cpu_baseline:
            # the checker runs the same chain S_l = 0.5 S_l + 0.5 S_{l-1} on its own scores for the sampled heads
            from oracle import critiprefill_oracle as O
            prev, recs = None, []
            step()                                              # outputs and lists of all layers of this budget
            torch.cuda.synchronize()
            for l, (q_h, k_h, v_h) in enumerate(host):
                rec, prev = cpu_baseline_layer(O, synth, np, wb, q_h, k_h, v_h, lists[l][0], lists[l][1], out[l],
                                               max(2, args.cpu_heads // 2), max(8, args.cpu_segments // 40),
                                               prev=prev, alpha=w.alpha)
                recs.append(rec)
            errs = [r["sampled_output_max_abs_err"] for r in recs if r["sampled_output_max_abs_err"] is not None]
            result["cpu_baseline"] = {
                "value": round(sum(r["value"] for r in recs), 1), "unit": "ms",
                "cores": round(float(np.mean([r["cores"] for r in recs])), 1), "kind": "oracle",
                "threads": cpu_threads(),
                "sample": f"sum over {w.layers} layers; per layer: " + recs[0]["sample"],
                "sampled_segments_compared": sum(r["sampled_segments_compared"] for r in recs),
                "sampled_segments_total": sum(r["sampled_segments_total"] for r in recs),
                "sampled_output_max_abs_err": max(errs) if errs else None,
            }
        print(json.dumps(result), flush=True)
        del lists


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10,
                    help="untimed steps; the attention kernel keeps getting faster over the first ~8 launches after an idle phase")
    ap.add_argument("--workload", default="c3_llama3_8b_128k")
    ap.add_argument("--dense-steps", type=int, default=3)
    ap.add_argument("--budgets", default="512,1024,4096", help="token budgets of the multi-layer workload, one JSON line each")
    ap.add_argument("--rotate", type=int, default=0, help="copies of the inputs to rotate over (0: 4 when one copy is near the Infinity Cache size, else 1)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy (a known-size kernel to scale rocprofv3 FETCH_SIZE/WRITE_SIZE by)")
    ap.add_argument("--cpu-heads", type=int, default=8, help="(batch, head) pairs the CPU checker estimates, selects and attends")
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
    if w.layers > 1:
        run_stack(args, np, torch, B, synth, w, dev)
    else:
        run_single_layer(args, np, torch, B, synth, w, dev)
    return 0


if __name__ == "__main__":
    sys.exit(main())
