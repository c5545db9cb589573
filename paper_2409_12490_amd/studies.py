#!/usr/bin/env python3
"""Four measurements beyond the headline benchmark, on one MI355X, printed as JSON lines.

``python -m paper_2409_12490_amd.studies fusion``
    Cost of the layer-fusion line of Algorithm 1 (S = alpha*S + (1-alpha)*S'): the estimate step at 128K with and
    without the previous layer's scores, for alpha in {0.25 (the paper's experiments section), 0.5, 1.0}.  The paper's
    ablation says that fusion changes quality, not speed; this measures the speed half of that statement.

``python -m paper_2409_12490_amd.studies length``
    Latency of one layer against sequence length, 8K .. 128K, at the hyper-parameters of the paper's experiments
    section (segment 512, block 32, budget 1024 tokens) and at the benchmark's block size 64: estimate + select +
    block-sparse attention against the library's dense causal kernel.  The build's analogue of the paper's
    prefill-time-against-length figure (quadratic against linear growth).

``python -m paper_2409_12490_amd.studies locality``
    The locality that the method rests on (its Eq. 3 and the overlap heat map next to it), on the generator's data at
    16K tokens: (i) overlap |K_i ∩ K_j| / k of the exact per-query top-k token sets of queries i and j = i + delta, for
    delta = 1 .. 4096; (ii) how much of a query's exact top-k set, and of its softmax mass, the block lists of the
    library (estimate + select) retain, against lists of the same size made of the most recent blocks only.  A
    quality proxy that needs no dataset and no trained weights.  A query's exact set is the top-k of q.k among the
    strictly earlier keys plus its own position (the convention of the path: the diagonal is always attended); the
    sets come from plain torch operations on the GPU (a dense score matrix and ``topk``) and are checked against the
    CPU checker's own per-query top-k (segment = block = 1) in tests/test_gpu_studies.py; the block lists come from
    the library.

``python -m paper_2409_12490_amd.studies shared``
    One block list per KV head (from the maximum of its query heads' scores) instead of one per query head, an
    extension the paper does not describe: latency of select + sparse attention and the change of the output error
    (against the library's dense kernel) at 128K, for the budget of the benchmark and for a budget G times larger
    (the union of G per-head lists is at most that long); on the Llama3-8B shape (4 query heads per KV head) and the
    Yi-9B shape (8 per KV head), the latter also with blocks of 32 tokens.

Inputs are the seeded synthetic Q/K/V of ``synth``; every latency and every block list comes from the HIP library
through the C ABI.
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


def exact_topk_members(qh: torch.Tensor, kh: torch.Tensor, topk: int, scale: float):
    """The exact critical set of every query of one head (Eq. 3 of the paper, with the convention the path itself
    uses): the ``topk`` keys with the largest q.k among the strictly earlier positions, plus the query's own
    position.  qh, kh: [n, d] float32 on the GPU.  Returns (member [n, n] bool, prob [n, n] float32 = the causal
    softmax of the scaled logits)."""
    n, dev = qh.shape[0], qh.device
    rows = torch.arange(n, device=dev)
    member = torch.zeros((n, n), dtype=torch.bool, device=dev)
    prob_rows = []
    kk = min(topk, n)
    for r0 in range(0, n, 2048):
        z = (qh[r0:r0 + 2048] @ kh.T) * scale
        zc = z.masked_fill(rows[None, :] > rows[r0:r0 + 2048, None], float("-inf"))
        prob_rows.append(torch.softmax(zc, dim=1))
        zs = z.masked_fill(rows[None, :] >= rows[r0:r0 + 2048, None], float("-inf"))
        top = zs.topk(kk, dim=1).indices
        member[r0:r0 + 2048].scatter_(1, top, True)
    member &= rows[None, :] < rows[:, None]                  # queries with fewer than topk earlier keys: drop the padding picks
    member |= rows[None, :] == rows[:, None]
    return member, torch.cat(prob_rows)


def locality(dev: str = "cuda:0", seq_len: int = 16384, heads=(0, 5, 10, 15, 20, 25, 30, 31), topk: int = 1024,
             keep_sets: dict | None = None) -> None:
    """keep_sets: optional dict that receives, per (setting label, head), the exact sets (bool [n, n], on the CPU)
    and the library's block lists, for checks against an independent implementation."""
    w = synth.WORKLOADS["c2_llama3_8b_16k"].replace(seq_len=seq_len, name=f"llama3_8b_{seq_len // 1024}k")
    q, k, _ = synth.make_qkv(w, threads=min(16, os.cpu_count() or 8))
    q, k = q.to(dev), k.to(dev)
    n, s, G = seq_len, w.segment_size, w.n_q_heads // w.n_kv_heads
    scale = 1.0 / (w.head_dim ** 0.5)
    deltas = [d for d in (1, 8, 64, 512, 4096) if d < n - topk]
    rows = torch.arange(n, device=dev)
    for label, b, budget_blocks, local in (("paper: s=512 b=32 B=1024", 32, 1024 // 32, 0),
                                           ("bench: s=512 b=64 B=2048 L=1", 64, 2048 // 64, 1)):
        p = B.make_params(q, k, s, b, budget_blocks, local)
        S, ws = B.alloc_scores(p, dev), B.alloc_workspace(p, dev)
        idx, cnt = B.alloc_lists(p, dev)
        B.critiprefill_estimate(p, q, k, None, S, ws)
        B.critiprefill_select(p, S, idx, cnt)
        torch.cuda.synchronize()
        n1, n2, r = w.n_segments, -(-n // b), s // b
        overlap = {d: [] for d in deltas}
        kept_set, kept_mass, recent_set, recent_mass = [], [], [], []
        for h in heads:
            member, prob = exact_topk_members(q[0, h].float(), k[0, h // G].float(), topk, scale)
            size = member.sum(1).float()                      # topk + 1 once a query has topk earlier keys
            full = rows >= topk
            for d in deltas:
                both = (member[:-d] & member[d:]).sum(1).float() / size[d:]
                overlap[d].append(float(both[full[:-d]].mean()))
            # what the block lists keep: tokens of the listed blocks, per segment; and the same number of most recent blocks
            tok_block = rows // b
            li = idx[0, h].long(); lc = cnt[0, h].long()
            valid = torch.arange(li.shape[1], device=dev)[None, :] < lc[:, None]
            # (added up, not assigned: the padding entries are clamped onto block 0 and must not unmark it)
            listed = torch.zeros((n1, n2), dtype=torch.int32, device=dev).scatter_add_(1, li.clamp(min=0), valid.int()) > 0
            seg = rows // s
            recent = torch.zeros((n1, n2), dtype=torch.bool, device=dev)
            blocks = torch.arange(n2, device=dev)
            last = (torch.arange(n1, device=dev) + 1) * r           # first block after the segment
            recent |= (blocks[None, :] < last[:, None]) & (blocks[None, :] >= (last - lc)[:, None])
            for mask_blocks, out_set, out_mass in ((listed, kept_set, kept_mass), (recent, recent_set, recent_mass)):
                tok_mask = mask_blocks[seg][:, tok_block]           # [query, token]: the token's block is in the query's list
                out_set.append(float(((member & tok_mask).sum(1).float() / size)[full].mean()))
                out_mass.append(float((prob * tok_mask).sum(1)[full].mean()))
            if keep_sets is not None:
                keep_sets[(label, h)] = {"member": member.cpu(), "idx": idx[0, h].cpu(), "cnt": cnt[0, h].cpu(),
                                         "block": b, "segment": s, "budget_blocks": budget_blocks, "local_blocks": local,
                                         "kept_of_set": kept_set[-1], "recent_of_set": recent_set[-1],
                                         "overlap": {d: overlap[d][-1] for d in deltas}}
            del member, prob
        mean = lambda xs: round(sum(xs) / len(xs), 4)
        print(json.dumps({"study": "locality", "seq_len": n, "setting": label, "heads": list(heads), "topk_tokens": topk,
                          "overlap_of_exact_topk_sets_by_query_distance": {str(d): mean(v) for d, v in overlap.items()},
                          "kept_by_block_lists": {"of_exact_topk_set": mean(kept_set), "of_softmax_mass": mean(kept_mass)},
                          "kept_by_most_recent_blocks_same_count": {"of_exact_topk_set": mean(recent_set),
                                                                     "of_softmax_mass": mean(recent_mass)},
                          "mean_listed_blocks": round(float(cnt[0, list(heads)].float().mean()), 2),
                          "blocks_total": n2}), flush=True)


def shared(dev: str = "cuda:0", workload: str = "c3_llama3_8b_128k", block_size: int = 0) -> None:
    w = synth.WORKLOADS[workload]
    if block_size:                                          # same token budget and local window in blocks of another size
        f = w.block_size // block_size
        w = w.replace(block_size=block_size, budget_blocks=w.budget_blocks * f, local_blocks=w.local_blocks * f)
    q, k, v = synth.make_qkv(w, threads=min(16, os.cpu_count() or 8))
    q, k, v = q.to(dev), k.to(dev), v.to(dev)
    out, dense = torch.empty_like(q), torch.empty_like(q)
    p0 = B.make_params(q, k, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks, out=out)
    B.critiprefill_dense_causal_attn(p0, q, k, v, dense, None)
    S, ws = B.alloc_scores(p0, dev), B.alloc_workspace(p0, dev)
    B.critiprefill_estimate(p0, q, k, None, S, ws)
    G = w.n_q_heads // w.n_kv_heads

    def err(o):
        d = (o.float() - dense.float())
        return float(d.abs().max()), float(d.norm() / dense.float().norm())

    for budget in (w.budget_blocks, G * w.budget_blocks):
        p = B.make_params(q, k, w.segment_size, w.block_size, budget, w.local_blocks, out=out)
        for kind in ("per query head", "per KV head"):
            if kind == "per query head":
                idx, cnt = B.alloc_lists(p, dev)
                sel = lambda: B.critiprefill_select(p, S, idx, cnt)
                att = lambda: B.critiprefill_sparse_attn(p, q, k, v, idx, cnt, out, None)
            else:
                idx, cnt = B.alloc_shared_lists(p, dev)
                sel = lambda: B.critiprefill_select_shared(p, S, idx, cnt)
                att = lambda: B.critiprefill_sparse_attn_shared(p, q, k, v, idx, cnt, out, None)
            sel(); att(); torch.cuda.synchronize()
            e_max, e_rel = err(out)
            print(json.dumps({"study": "shared", "workload": w.name, "block_size": w.block_size, "group": G, "lists": kind, "budget_blocks": budget,
                              "select_ms": round(_time(sel, 10), 4), "sparse_attn_ms": round(_time(att, 10), 4),
                              "max_abs_vs_dense": round(e_max, 4), "rel_l2_vs_dense": round(e_rel, 5),
                              "mean_listed_blocks": round(float(cnt.float().mean()), 2)}), flush=True)


def main(argv) -> int:
    if len(argv) != 2 or argv[1] not in ("fusion", "length", "locality", "shared"):
        print(__doc__)
        return 2
    if not torch.cuda.is_available():
        print("studies: no GPU visible", file=sys.stderr)
        return 2
    B.load()
    torch.cuda.set_device(0)
    if argv[1] == "shared":
        # group 4 and 8, block 64 and 32: is the gather of K/V tiles per query head (instead of once per KV head) a cost?
        for workload, block in (("c3_llama3_8b_128k", 0), ("c4_yi_9b_128k", 0), ("c4_yi_9b_128k", 32)):
            shared(workload=workload, block_size=block)
        return 0
    {"fusion": fusion, "length": length, "locality": locality}[argv[1]]()
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
