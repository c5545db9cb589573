"""Shared test plumbing: run one workload through the HIP library (via the C ABI binding) and
through the CPU checker, and the comparison rules.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from oracle import critiprefill_oracle as O
from paper_2409_12490_amd import binding as B
from paper_2409_12490_amd import synth

TOL_OUT = {"bf16": 2e-2, "fp32": 1e-4}          # max-abs error of attention outputs vs the fp64 checker
TIE_BAND = 1e-3                                  # relative band around the k-th score inside which picks may differ


def params_for(w: synth.Workload, q, k, out=None, **kw):
    return B.make_params(q, k, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks, out=out,
                         alpha=w.alpha, **kw)


def gpu_estimate(w, q, k, prev=None, **kw):
    p = params_for(w, q, k, **kw)
    S = B.alloc_scores(p)
    ws = B.alloc_workspace(p)
    B.critiprefill_estimate(p, q, k, prev, S, ws)
    torch.cuda.synchronize()
    return S


def gpu_select(w, q, k, S):
    p = params_for(w, q, k)
    idx, cnt = B.alloc_lists(p)
    idx.fill_(-7)
    B.critiprefill_select(p, S, idx, cnt)
    torch.cuda.synchronize()
    return idx, cnt


def gpu_sparse(w, q, k, v, idx, cnt, want_lse=True, **kw):
    out = torch.full_like(q, float("nan"))
    p = params_for(w, q, k, out=out, **kw)
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device=q.device) if want_lse else None
    B.critiprefill_sparse_attn(p, q, k, v, idx, cnt, out, lse)
    torch.cuda.synchronize()
    return out, lse


def gpu_select_shared(w, q, k, S):
    p = params_for(w, q, k)
    idx, cnt = B.alloc_shared_lists(p)
    idx.fill_(-7)
    B.critiprefill_select_shared(p, S, idx, cnt)
    torch.cuda.synchronize()
    return idx, cnt


def gpu_sparse_shared(w, q, k, v, idx, cnt, **kw):
    out = torch.full_like(q, float("nan"))
    p = params_for(w, q, k, out=out, **kw)
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device=q.device)
    B.critiprefill_sparse_attn_shared(p, q, k, v, idx, cnt, out, lse)
    torch.cuda.synchronize()
    return out, lse


def gpu_dense(w, q, k, v, want_lse=True, **kw):
    out = torch.full_like(q, float("nan"))
    p = params_for(w, q, k, out=out, **kw)
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device=q.device) if want_lse else None
    B.critiprefill_dense_causal_attn(p, q, k, v, out, lse)
    torch.cuda.synchronize()
    return out, lse


def small_workload(name, B_, Hq, Hkv, n, s, b, k, L, dtype="bf16", seed=7, **kw):
    return synth.Workload(name, B_, Hq, Hkv, 128, n, s, b, k, L, dtype=dtype, seed=seed, **kw)


def check_selection(S_dec, idx_o, cnt_o, idx_g, cnt_g, w: synth.Workload, exact: bool, kth_floor: float = 0.0):
    """Compare block lists.  exact: bit-for-bit.  Otherwise the tie rule: the fixed (local + diagonal)
    part is identical, the counts are equal, every checker pick above the band around the k-th score
    is present, and no GPU pick lies below the band.  ``S_dec`` holds the scores the checker ranked.
    Rows whose k-th score is below ``kth_floor`` are only checked for structure (used when ranking the
    checker's unrounded fp64 scores: below the smallest normal fp32 the library's scores are flushed
    to zero and the order among them is the index order)."""
    idx_g = idx_g.cpu().numpy() if hasattr(idx_g, "cpu") else idx_g
    cnt_g = cnt_g.cpu().numpy() if hasattr(cnt_g, "cpu") else cnt_g
    np.testing.assert_array_equal(cnt_g, cnt_o)
    if exact:
        np.testing.assert_array_equal(idx_g, idx_o)
        return 0
    r = w.blocks_per_segment
    differing = 0
    Bn, H, n1, _ = idx_o.shape
    for b in range(Bn):
        for h in range(H):
            for j in range(n1):
                c = cnt_o[b, h, j]
                lo, lg = idx_o[b, h, j, :c], idx_g[b, h, j, :c]
                assert (idx_g[b, h, j, c:] == -1).all()
                if np.array_equal(lo, lg):
                    continue
                differing += 1
                n_cand = j * r - min(w.local_blocks, j * r)
                po, pg = lo[lo < n_cand], lg[lg < n_cand]
                np.testing.assert_array_equal(lo[lo >= n_cand], lg[lg >= n_cand])
                assert len(po) == len(pg) and (np.diff(lg) > 0).all()
                row = S_dec[b, h, j].astype(np.float64)
                kth = row[po].min()
                if kth < kth_floor:
                    continue
                band_hi, band_lo = kth * (1 + TIE_BAND), kth * (1 - TIE_BAND)
                must = po[row[po] > band_hi]
                assert np.isin(must, pg).all(), f"row {(b, h, j)}: a clear winner is missing"
                assert (row[pg] >= band_lo).all(), f"row {(b, h, j)}: a pick lies below the tie band"
    return differing


def max_abs(a, b):
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64))))
