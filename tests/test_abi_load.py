"""CPU-side checks of the boundary: the library loads, exports every function the header declares,
and rejects bad arguments before any kernel launch (no GPU needed for these paths)."""
import ctypes
import os
import re

import pytest

from paper_2409_12490_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "critiprefill.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(critiprefill_\w+)\s*\(", text)))


def test_header_functions_are_exported():
    if not os.path.exists(B.lib_path()):
        import paper_2409_12490_amd.build as build
        build.build()
    lib = B.load()
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None
    assert B.version() >= 200
    assert B.strerror(0) == "ok"


def _params(**kw):
    p = B.Params()
    p.batch, p.n_q_heads, p.n_kv_heads, p.head_dim = 1, 4, 2, 128
    p.seq_len, p.segment_size, p.block_size, p.budget_blocks, p.local_blocks = 1024, 128, 32, 4, 1
    p.dtype = B.CP_DTYPE_BF16
    for i, s in enumerate((4 * 1024 * 128, 1024 * 128, 128)):
        p.q_stride[i] = s; p.o_stride[i] = s
    for i, s in enumerate((2 * 1024 * 128, 1024 * 128, 128)):
        p.kv_stride[i] = s
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_sizes():
    p = _params()
    assert B.critiprefill_list_len(p) == 4 + 1 + 4
    n1, n2 = 8, 32
    # representatives of 4 query heads x n1 segments and 2 KV heads x n2 blocks, then the score statistics of the
    # bf16 path: per head and chunk of 256 blocks (one chunk here, cut in 8 parts because a sequence of at most 16
    # segments lets the 8 waves of a workgroup share them), 2 products x (max, sum) x 2 representatives x 128-padded segments
    assert B.critiprefill_workspace_bytes(p) == (4 * n1 + 2 * n2) * 2 * 128 * 2 + 4 * (1 * 8) * 2 * 2 * (2 * 128) * 4
    p = _params(dtype=B.CP_DTYPE_FP32, seq_len=1000)
    n1, n2 = 8, 32
    assert B.critiprefill_workspace_bytes(p) == (4 * n1 + 2 * n2) * 2 * 128 * 4


@pytest.mark.parametrize("kw,code", [
    (dict(batch=0), -2), (dict(n_kv_heads=3), -2), (dict(block_size=48), -2), (dict(seq_len=-5), -2),
    (dict(head_dim=64), -3), (dict(dtype=7), -3), (dict(softmax_domain=2), -3), (dict(attn_scale=-1.0), -2),
])
def test_bad_shapes_are_rejected_before_launch(kw, code):
    lib = B.load()
    p = _params(**kw)
    fake = ctypes.c_void_p(0x1000)        # never dereferenced: the shape check fails first
    assert lib.critiprefill_estimate(ctypes.byref(p), fake, fake, None, fake, fake, 1 << 30, None) == code
    assert lib.critiprefill_estimate_static(ctypes.byref(p), fake, fake, None, fake, None) == code
    assert lib.critiprefill_select(ctypes.byref(p), fake, fake, fake, None) == code
    assert lib.critiprefill_sparse_attn(ctypes.byref(p), fake, fake, fake, fake, fake, fake, None, None) == code
    assert lib.critiprefill_dense_causal_attn(ctypes.byref(p), fake, fake, fake, fake, None, None) == code
    assert B.critiprefill_list_len(p) == code
    assert lib.critiprefill_select_shared(ctypes.byref(p), fake, fake, fake, None) == code
    assert lib.critiprefill_sparse_attn_shared(ctypes.byref(p), fake, fake, fake, fake, fake, fake, None, None) == code
    assert B.critiprefill_workspace_bytes(p) == 0


def test_bf16_estimate_rejects_more_than_65535_batch_heads():
    lib = B.load()
    p = _params(batch=16384)                # 16384 * 4 query heads
    fake = ctypes.c_void_p(0x1000)
    assert lib.critiprefill_estimate(ctypes.byref(p), fake, fake, None, fake, fake, 1 << 40, None) == -3


def test_null_alignment_and_workspace_errors():
    lib = B.load()
    p = _params()
    ok, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    assert lib.critiprefill_estimate(None, ok, ok, None, ok, ok, 1 << 30, None) == -1
    assert lib.critiprefill_estimate(ctypes.byref(p), None, ok, None, ok, ok, 1 << 30, None) == -1
    assert lib.critiprefill_estimate(ctypes.byref(p), odd, ok, None, ok, ok, 1 << 30, None) == -4
    assert lib.critiprefill_estimate(ctypes.byref(p), ok, ok, None, ok, ok, 16, None) == -5
    assert lib.critiprefill_estimate_static(ctypes.byref(p), ok, None, None, ok, None) == -1
    assert lib.critiprefill_estimate_static(ctypes.byref(p), ok, ok, odd, ok, None) == -4
    big = _params(n_q_heads=64, n_kv_heads=64, seq_len=131072, segment_size=512, block_size=16)   # needs > 32 MiB of scratch
    assert B.critiprefill_workspace_bytes(big) > (32 << 20)
    assert lib.critiprefill_estimate_static(ctypes.byref(big), ok, ok, None, ok, None) == -5
    assert lib.critiprefill_select(ctypes.byref(p), ok, None, ok, None) == -1
    assert lib.critiprefill_select(ctypes.byref(p), ok, odd, ok, None) == -4
    assert lib.critiprefill_sparse_attn(ctypes.byref(p), ok, ok, ok, None, ok, ok, None, None) == -1
    assert lib.critiprefill_sparse_attn(ctypes.byref(p), ok, ok, odd, ok, ok, ok, None, None) == -4
    assert lib.critiprefill_dense_causal_attn(ctypes.byref(p), ok, ok, ok, None, None, None) == -1
    q = _params(); q.q_stride[2] = 132
    assert lib.critiprefill_dense_causal_attn(ctypes.byref(q), ok, ok, ok, ok, None, None) == -4
    q = _params(seq_len=8192 * 32 + 1)
    assert lib.critiprefill_select(ctypes.byref(q), ok, ok, ok, None) == -3
    with pytest.raises(B.CritiPrefillError):
        B._check(-3, "x")
