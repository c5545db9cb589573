"""critiprefill_estimate_static (the entry point for callers that cannot allocate: scratch in a fixed device array
inside the library) against critiprefill_estimate (scratch in the caller's workspace), through the C ABI.

Same kernels on the same inputs, so the scores must be bit-identical.  Two calls in a row on the shared array,
the second on a smaller input (the array keeps the first call's contents), plus the size limit.
"""
import ctypes

import pytest
import torch

from paper_2409_12490_amd import binding as B
from paper_2409_12490_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def both_ways(w, prev_seed=None):
    q, k, _ = synth.make_qkv(w, threads=4)
    q, k = q.to(DEV), k.to(DEV)
    p = H.params_for(w, q, k)
    prev = None
    if prev_seed is not None:
        g = torch.Generator(device="cpu").manual_seed(prev_seed)
        prev = torch.rand((w.batch, w.n_q_heads, w.n_segments, w.n_blocks), generator=g).to(DEV)
    S_ws = B.alloc_scores(p).fill_(float("nan"))
    B.critiprefill_estimate(p, q, k, prev, S_ws, B.alloc_workspace(p))
    S_st = B.alloc_scores(p).fill_(float("nan"))
    B.critiprefill_estimate_static(p, q, k, prev, S_st)
    torch.cuda.synchronize()
    return S_ws, S_st


def test_static_scratch_matches_workspace_twice_second_smaller():
    big = H.small_workload("static_big", 1, 4, 2, 8400, 64, 16, 6, 1)            # several score chunks, ragged tail
    small = H.small_workload("static_small", 1, 2, 1, 1000, 128, 32, 4, 0, alpha=0.25)
    print("first call:", big.name, flush=True)
    S_ws, S_st = both_ways(big)
    assert torch.isfinite(S_st).all() and torch.equal(S_ws, S_st)
    print("second call (smaller, with layer fusion):", small.name, flush=True)
    S_ws, S_st = both_ways(small, prev_seed=1)
    assert torch.isfinite(S_st).all() and torch.equal(S_ws, S_st)
    print("third call (fp32):", flush=True)
    S_ws, S_st = both_ways(H.small_workload("static_fp32", 1, 2, 1, 700, 128, 32, 4, 0, dtype="fp32", unit_variance=False))
    assert torch.isfinite(S_st).all() and torch.equal(S_ws, S_st)


def test_static_scratch_rejects_sizes_beyond_its_limit():
    # 64 query heads x 128K tokens in blocks of 16: the K representatives alone need more than 32 MiB
    w = synth.Workload("too_big", 1, 64, 64, 128, 131072, 512, 16, 8, 0)
    q = torch.empty((1, 1, 16, 128), dtype=torch.bfloat16, device=DEV)            # never read: the check fails first
    p = B.Params()
    p.batch, p.n_q_heads, p.n_kv_heads, p.head_dim, p.seq_len = 1, 64, 64, 128, w.seq_len
    p.segment_size, p.block_size, p.budget_blocks, p.local_blocks, p.dtype = 512, 16, 8, 0, B.CP_DTYPE_BF16
    for i, s in enumerate((64 * w.seq_len * 128, w.seq_len * 128, 128)):
        p.q_stride[i] = s; p.kv_stride[i] = s; p.o_stride[i] = s
    assert B.critiprefill_workspace_bytes(p) > (32 << 20)
    st = B.load().critiprefill_estimate_static(ctypes.byref(p), ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(q.data_ptr()),
                                               None, ctypes.c_void_p(q.data_ptr()), None)
    assert st == -5
