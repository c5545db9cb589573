#!/usr/bin/env python3
"""Two measurements beyond the headline benchmark, on one MI355X, printed as JSON lines.

``python -m paper_2409_12490_amd.studies fusion``
    Cost of the layer-fusion line of Algorithm 1 (S = alpha*S + (1-alpha)*S'): the estimate step at 128K with and
    without the previous layer's scores, for alpha in {0.25 (the paper's experiments section), 0.5, 1.0}.  The paper's
    ablation says that fusion changes quality, not speed; this measures the speed half of that statement.

``python -m paper_2409_12490_amd.studies length``
    Latency of one layer against sequence length, 8K .. 128K, at the hyper-parameters of the paper's experiments
    section (segment 512, block 32, budget 1024 tokens) and at the benchmark's block size 64: estimate + select +
    block-sparse attention against the library's dense causal kernel.  The build's analogue of the paper's
    prefill-time-against-length figure (quadratic against linear growth).

Inputs are the seeded synthetic Q/K/V of ``synth``; every number comes from the HIP library through the C ABI.
"""
from __future__ import annotations

import json
import os
import sys

import torch

from . import binding as B
from . import synth


def _time(fn, steps: int) -> float:
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def fusion(dev: str = "cuda:0") -> None:
    w = synth.WORKLOADS["c3_llama3_8b_128k"]
    q, k, _ = synth.make_qkv(w, threads=min(16, os.cpu_count() or 8))
    q, k = q.to(dev), k.to(dev)
    p = B.make_params(q, k, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks)
    ws = B.alloc_workspace(p, dev)
    prev, cur = B.alloc_scores(p, dev), B.alloc_scores(p, dev)
    B.critiprefill_estimate(p, q, k, None, prev, ws)                 # stands in for the previous layer's S'
    base = _time(lambda: B.critiprefill_estimate(p, q, k, None, cur, ws), 20)
    for alpha in (0.25, 0.5, 1.0):
        pa = B.make_params(q, k, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks, alpha=alpha)
        fused = _time(lambda: B.critiprefill_estimate(pa, q, k, prev, cur, ws), 20)
        print(json.dumps({"study": "fusion", "workload": w.name, "alpha": alpha,
                          "estimate_ms_without_prev": round(base, 4), "estimate_ms_with_prev": round(fused, 4),
                          "delta_ms": round(fused - base, 4),
                          "extra_bytes_read": int(prev.numel() * 4)}), flush=True)


def length(dev: str = "cuda:0") -> None:
    w0 = synth.WORKLOADS["c3_llama3_8b_128k"]
    for n in (8192, 16384, 32768, 65536, 131072):
        wn = w0.replace(seq_len=n, name=f"llama3_8b_{n // 1024}k")
        q, k, v = synth.make_qkv(wn, threads=min(16, os.cpu_count() or 8))
        q, k, v = q.to(dev), k.to(dev), v.to(dev)
        out = torch.empty_like(q)
        dense_steps = 3 if n >= 65536 else 10
        p_d = B.make_params(q, k, 512, 64, 32, 1, out=out)
        dense = _time(lambda: B.critiprefill_dense_causal_attn(p_d, q, k, v, out, None), dense_steps)
        for label, b, budget_blocks, local in (("paper: s=512 b=32 B=1024", 32, 32, 0),
                                               ("bench: s=512 b=64 B=2048 L=1", 64, 32, 1)):
            p = B.make_params(q, k, 512, b, budget_blocks, local, out=out)
            S, ws = B.alloc_scores(p, dev), B.alloc_workspace(p, dev)
            idx, cnt = B.alloc_lists(p, dev)

            def step():
                B.critiprefill_estimate(p, q, k, None, S, ws)
                B.critiprefill_select(p, S, idx, cnt)
                B.critiprefill_sparse_attn(p, q, k, v, idx, cnt, out, None)

            total = _time(step, 10)
            est = _time(lambda: B.critiprefill_estimate(p, q, k, None, S, ws), 10)
            sel = _time(lambda: B.critiprefill_select(p, S, idx, cnt), 10)
            att = _time(lambda: B.critiprefill_sparse_attn(p, q, k, v, idx, cnt, out, None), 10)
            print(json.dumps({"study": "length", "seq_len": n, "setting": label,
                              "layer_ms": round(total, 4), "estimate_ms": round(est, 4), "select_ms": round(sel, 4),
                              "sparse_attn_ms": round(att, 4), "dense_causal_ms": round(dense, 4),
                              "speedup_vs_dense": round(dense / total, 3)}), flush=True)
        del q, k, v, out


def main(argv) -> int:
    if len(argv) != 2 or argv[1] not in ("fusion", "length"):
        print(__doc__)
        return 2
    if not torch.cuda.is_available():
        print("studies: no GPU visible", file=sys.stderr)
        return 2
    B.load()
    torch.cuda.set_device(0)
    {"fusion": fusion, "length": length}[argv[1]]()
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
