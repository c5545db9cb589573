"""GPU parity: every entry point of the C ABI against the fp64 CPU checker on the same seeded inputs.

Bars: block lists bit-exact when both sides rank the same fp32 scores; end to end (GPU scores vs
checker scores) equal outside a 1e-3 relative tie band around the k-th score; attention outputs
max-abs <= 2e-2 (bf16) / 1e-4 (fp32).
"""
import numpy as np
import pytest
import torch

from oracle import critiprefill_oracle as O
from paper_2409_12490_amd import binding as B
from paper_2409_12490_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda"

SMALL = [
    # name                    B Hq Hkv   n    s    b  k  L  dtype
    ("bf16_ragged_b64",       1, 4, 2, 1500, 256,  64, 4, 1, "bf16"),
    ("bf16_b32_gqa4",         2, 4, 1, 1024, 128,  32, 6, 0, "bf16"),
    ("bf16_b16_small_seg",    1, 2, 2,  777,  64,  16, 5, 2, "bf16"),
    ("bf16_b128_seg512",      1, 2, 1, 2048, 512, 128, 3, 1, "bf16"),
    ("bf16_seg_eq_block",     1, 2, 2,  640,  64,  64, 2, 1, "bf16"),
    ("bf16_many_segments",    1, 2, 1, 8400,  64,  16, 6, 1, "bf16"),   # 132 segments, 525 blocks: several score chunks
    ("fp32_c1_like",          1, 2, 1, 1000, 128,  32, 8, 0, "fp32"),
    ("fp32_b8",               1, 3, 3,  300,  32,   8, 4, 1, "fp32"),
]


def make(case, **kw):
    name, B_, Hq, Hkv, n, s, b, k, L, dtype = case
    w = H.small_workload(name, B_, Hq, Hkv, n, s, b, k, L, dtype=dtype, unit_variance=(dtype == "bf16"), **kw)
    q, k_, v = synth.make_qkv(w, threads=4)
    return w, q, k_, v


def oracle_lists(w, q, k):
    S = O.estimate(synth.to_f64(q), synth.to_f64(k), w.segment_size, w.block_size)
    Sd = O.scores_in_decision_precision(S)
    idx, cnt = O.select(Sd, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks)
    return S, Sd, idx, cnt


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_estimate_scores(case):
    w, q, k, v = make(case)
    print("case", case, flush=True)
    qf, kf = synth.to_f64(q), synth.to_f64(k)
    for domain in (0, 1):
        S_o = O.estimate(qf, kf, w.segment_size, w.block_size, softmax_domain=domain)
        S_g = H.gpu_estimate(w, q.to(DEV), k.to(DEV), softmax_domain=domain).cpu().numpy()
        np.testing.assert_allclose(S_g, S_o, rtol=2e-4, atol=1e-30)
    # another scale, then the listing taken literally (score_scale = 1.0: no 1/sqrt(d); logits of the max/min
    # representatives reach the hundreds, so each softmax is nearly one-hot and most scores underflow to 0)
    S_o = O.estimate(qf, kf, w.segment_size, w.block_size, score_scale=0.05)
    S_g = H.gpu_estimate(w, q.to(DEV), k.to(DEV), score_scale=0.05).cpu().numpy()
    np.testing.assert_allclose(S_g, S_o, rtol=2e-4, atol=1e-30)
    S_o = O.scores_in_decision_precision(O.estimate(qf, kf, w.segment_size, w.block_size, score_scale=1.0))
    S_g = H.gpu_estimate(w, q.to(DEV), k.to(DEV), score_scale=1.0).cpu().numpy()
    # a logit z carries an fp32 rounding error of about |z| 2^-23 (accumulation of 128 exact products), which
    # the exponential turns into a relative error of the same size in the score: |z| up to ~1e3 -> ~2e-4
    np.testing.assert_allclose(S_g, S_o, rtol=1e-3, atol=2e-38)
    prev = np.random.default_rng(0).random(S_o.shape).astype(np.float32)
    S_f = O.estimate(qf, kf, w.segment_size, w.block_size, prev_scores=prev.astype(np.float64), alpha=0.25)
    w2 = w.replace(alpha=0.25)
    S_g = H.gpu_estimate(w2, q.to(DEV), k.to(DEV), prev=torch.from_numpy(prev).to(DEV)).cpu().numpy()
    np.testing.assert_allclose(S_g, S_f, rtol=2e-4, atol=1e-30)


def test_estimate_fusion_in_place():
    """prev_scores may alias scores (the fused score of the previous layer is overwritten by this layer's)."""
    case = [c for c in SMALL if c[0] == "bf16_many_segments"][0]
    w, q, k, v = make(case)
    w = w.replace(alpha=0.5)
    qf, kf = synth.to_f64(q), synth.to_f64(k)
    prev = np.random.default_rng(3).random((w.batch, w.n_q_heads, w.n_segments, w.n_blocks)).astype(np.float32)
    S_o = O.estimate(qf, kf, w.segment_size, w.block_size, prev_scores=prev.astype(np.float64), alpha=0.5)
    p = H.params_for(w, q.to(DEV), k.to(DEV))
    S = torch.from_numpy(prev).to(DEV)
    ws = B.alloc_workspace(p)
    B.critiprefill_estimate(p, q.to(DEV), k.to(DEV), S, S, ws)
    torch.cuda.synchronize()
    np.testing.assert_allclose(S.cpu().numpy(), S_o, rtol=2e-4, atol=1e-30)


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_select_bit_exact_on_same_scores(case):
    w, q, k, v = make(case)
    print("case", case, flush=True)
    S, Sd, idx_o, cnt_o = oracle_lists(w, q, k)
    Sd = Sd.copy()
    # plant exact ties and zeros so the tie-break and the k-th = 0 case are exercised
    Sd[..., 1::3] = Sd[..., 0:-1:3][..., :Sd[..., 1::3].shape[-1]]
    Sd[:, :, -1, : Sd.shape[-1] // 2] = 0.0
    idx_o, cnt_o = O.select(Sd, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks)
    idx_g, cnt_g = H.gpu_select(w, q.to(DEV), k.to(DEV), torch.from_numpy(Sd).to(DEV))
    H.check_selection(Sd, idx_o, cnt_o, idx_g, cnt_g, w, exact=True)


def test_select_negative_and_large_budget():
    w = H.small_workload("sel", 1, 2, 1, 4096, 64, 16, 300, 3)
    g = np.random.default_rng(5)
    Sd = (g.standard_normal((1, 2, w.n_segments, w.n_blocks)) * 1e-3).astype(np.float32)   # fused scores may be any sign
    idx_o, cnt_o = O.select(Sd, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks)
    q = torch.empty((1, 2, w.seq_len, 128), dtype=torch.bfloat16, device=DEV)
    k = torch.empty((1, 1, w.seq_len, 128), dtype=torch.bfloat16, device=DEV)
    idx_g, cnt_g = H.gpu_select(w, q, k, torch.from_numpy(Sd).to(DEV))
    H.check_selection(Sd, idx_o, cnt_o, idx_g, cnt_g, w, exact=True)


@pytest.mark.parametrize("n_blocks,budget", [(4096, 32), (8192, 100)])
def test_select_long_rows_with_ties(n_blocks, budget):
    """Rows of 4096 blocks (64 per lane) and 8192 blocks (one workgroup per row), scores quantised to a handful of
    levels so that the k-th score is shared by hundreds of blocks and the smallest-index tie rule decides."""
    b = 16
    w = H.small_workload("long", 1, 2, 1, n_blocks * b, 512, b, budget, 2)
    g = np.random.default_rng(n_blocks)
    Sd = (g.integers(0, 7, size=(1, 2, w.n_segments, w.n_blocks)) / 8.0).astype(np.float32)
    Sd[:, :, :, 5::11] += g.random(Sd[:, :, :, 5::11].shape, dtype=np.float32) * 1e-3     # a few distinct values too
    idx_o, cnt_o = O.select(Sd, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks)
    q = torch.empty((1, 2, w.seq_len, 128), dtype=torch.bfloat16, device=DEV)
    k = torch.empty((1, 1, w.seq_len, 128), dtype=torch.bfloat16, device=DEV)
    idx_g, cnt_g = H.gpu_select(w, q, k, torch.from_numpy(Sd).to(DEV))
    H.check_selection(Sd, idx_o, cnt_o, idx_g, cnt_g, w, exact=True)


@pytest.mark.parametrize("budget", [1, 32, 64, 128, 129])
@pytest.mark.parametrize("layout", ["spread", "one_lane", "few_distinct"])
def test_select_rows_of_2048_blocks(budget, layout):
    """Rows of up to 2048 candidates with distinct scores: large scores spread over the row, large scores only at
    block indices = 5 mod 64 (all in one lane of the kernel's wave, so that thinning the row by per-lane maxima
    keeps too many candidates and the kernel must search the whole row), and a row whose large scores are few."""
    b = 64
    w = H.small_workload("sel2k", 1, 2, 1, 2048 * b, 512, b, budget, 1)
    g = np.random.default_rng(100 * budget + len(layout))
    Sd = g.random((1, 2, w.n_segments, w.n_blocks), dtype=np.float32) * 1e-3
    if layout == "one_lane":
        Sd[..., 5::64] += 1.0
    elif layout == "few_distinct":
        Sd[..., ::97] += 0.5
    idx_o, cnt_o = O.select(Sd, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks)
    q = torch.empty((1, 2, w.seq_len, 128), dtype=torch.bfloat16, device=DEV)
    k = torch.empty((1, 1, w.seq_len, 128), dtype=torch.bfloat16, device=DEV)
    idx_g, cnt_g = H.gpu_select(w, q, k, torch.from_numpy(Sd).to(DEV))
    H.check_selection(Sd, idx_o, cnt_o, idx_g, cnt_g, w, exact=True)


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_estimate_then_select_tie_band(case):
    w, q, k, v = make(case)
    print("case", case, flush=True)
    S, Sd, idx_o, cnt_o = oracle_lists(w, q, k)
    S_g = H.gpu_estimate(w, q.to(DEV), k.to(DEV))
    idx_g, cnt_g = H.gpu_select(w, q.to(DEV), k.to(DEV), S_g)
    H.check_selection(Sd, idx_o, cnt_o, idx_g, cnt_g, w, exact=False)


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_sparse_attention_with_checker_lists(case):
    w, q, k, v = make(case)
    print("case", case, flush=True)
    _, _, idx_o, cnt_o = oracle_lists(w, q, k)
    o_ref, lse_ref = O.sparse_attention(synth.to_f64(q), synth.to_f64(k), synth.to_f64(v), idx_o, cnt_o,
                                        w.segment_size, w.block_size)
    out, lse = H.gpu_sparse(w, q.to(DEV), k.to(DEV), v.to(DEV),
                            torch.from_numpy(idx_o).to(DEV), torch.from_numpy(cnt_o).to(DEV))
    err = H.max_abs(out.float().cpu().numpy(), o_ref)
    print("max abs err", err, flush=True)
    assert err <= H.TOL_OUT[w.dtype]
    assert H.max_abs(lse.cpu().numpy(), lse_ref) <= (2e-2 if w.dtype == "bf16" else 1e-4)


@pytest.mark.parametrize("shape", [(4, 1, 35700, 512, 64), (2, 2, 66000, 256, 32), (3, 1, 70000, 1024, 64)],
                         ids=["280_pairs_2_tiles", "516_pairs_1_tile", "207_pairs_4_tiles"])
def test_sparse_attention_workgroup_order_covers_every_item(shape):
    """More (head, segment) pairs than one round of 256 workgroups holds, plus a remainder, at 1, 2 and 4 query tiles
    per segment: every output row is written (the output starts as NaN) and sampled segments, among them those around
    the border between the full rounds and the remainder, match the checker."""
    Hq, Hkv, n, s, b = shape
    w = H.small_workload("order", 1, Hq, Hkv, n, s, b, 4, 1)
    q, k, v = synth.make_qkv(w, threads=8)
    g = np.random.default_rng(3)
    Sd = g.random((1, Hq, w.n_segments, w.n_blocks), dtype=np.float32)       # any scores will do: the lists are the input here
    idx_o, cnt_o = O.select(Sd, s, b, w.budget_blocks, w.local_blocks)
    out, lse = H.gpu_sparse(w, q.to(DEV), k.to(DEV), v.to(DEV), torch.from_numpy(idx_o).to(DEV), torch.from_numpy(cnt_o).to(DEV))
    out = out.float().cpu().numpy()
    assert not np.isnan(out).any() and not np.isnan(lse.cpu().numpy()).any()
    G = Hq // Hkv
    border = 256 // G                                                       # segment of the first pair past one full round
    segs = sorted({0, 1, border - 1, border, border + 1, w.n_segments // 2, w.n_segments - 2, w.n_segments - 1} & set(range(w.n_segments)))
    todo = [(0, h, j) for h in range(Hq) for j in segs]
    o_ref, _ = O.sparse_attention(synth.to_f64(q), synth.to_f64(k), synth.to_f64(v), idx_o, cnt_o, s, b, segments=todo)
    for (_, h, j) in todo:
        rows = slice(j * s, min(n, (j + 1) * s))
        assert H.max_abs(out[0, h, rows], o_ref[0, h, rows]) <= 2e-2, (h, j)


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_shared_lists_per_kv_head(case):
    """One list per KV head from the maximum of the group's scores: selection bit-exact on the same fp32
    scores, attention with those lists against the checker run with the list handed to every head."""
    w, q, k, v = make(case)
    print("case", case, flush=True)
    _, Sd, _, _ = oracle_lists(w, q, k)
    Sg = O.shared_group_scores(Sd, w.n_kv_heads)
    idx_o, cnt_o = O.select(Sg, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks)
    idx_g, cnt_g = H.gpu_select_shared(w, q.to(DEV), k.to(DEV), torch.from_numpy(Sd).to(DEV))
    assert tuple(idx_g.shape) == idx_o.shape
    H.check_selection(Sg, idx_o, cnt_o, idx_g, cnt_g, w, exact=True)
    idx_h, cnt_h = O.expand_shared_lists(idx_o, cnt_o, w.n_q_heads)
    o_ref, lse_ref = O.sparse_attention(synth.to_f64(q), synth.to_f64(k), synth.to_f64(v), idx_h, cnt_h,
                                        w.segment_size, w.block_size)
    out, lse = H.gpu_sparse_shared(w, q.to(DEV), k.to(DEV), v.to(DEV), idx_g, cnt_g)
    err = H.max_abs(out.float().cpu().numpy(), o_ref)
    print("max abs err", err, flush=True)
    assert err <= H.TOL_OUT[w.dtype]
    assert H.max_abs(lse.cpu().numpy(), lse_ref) <= (2e-2 if w.dtype == "bf16" else 1e-4)


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_dense_causal_attention(case):
    w, q, k, v = make(case)
    print("case", case, flush=True)
    o_ref, lse_ref = O.dense_causal_attention(synth.to_f64(q), synth.to_f64(k), synth.to_f64(v))
    out, lse = H.gpu_dense(w, q.to(DEV), k.to(DEV), v.to(DEV))
    err = H.max_abs(out.float().cpu().numpy(), o_ref)
    print("max abs err", err, flush=True)
    assert err <= H.TOL_OUT[w.dtype]
    assert H.max_abs(lse.cpu().numpy(), lse_ref) <= (2e-2 if w.dtype == "bf16" else 1e-4)


@pytest.mark.parametrize("gain", [6.0, 0.05], ids=["peaked", "flat"])
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_attention_peaked_and_flat_logits(dtype, gain):
    """Logits far from the unit scale of the other cases.  gain 6 (q and k both times 6: logits 36 times
    larger, every row's softmax dominated by one or two keys, the running maximum moving again and again while
    the row walks its tiles); gain 0.05 (all weights nearly equal).  Sparse and dense kernels against the checker."""
    w = H.small_workload("gain", 1, 4, 2, 2500, 256, 64, 6, 1, dtype=dtype, unit_variance=True)
    q, k, v = synth.make_qkv(w, threads=2)
    q, k = (q.float() * gain).to(q.dtype), (k.float() * gain).to(k.dtype)
    print("dtype", dtype, "gain", gain, flush=True)
    qf, kf, vf = synth.to_f64(q), synth.to_f64(k), synth.to_f64(v)
    _, _, idx_o, cnt_o = oracle_lists(w, q, k)
    tol_lse = 2e-2 if dtype == "bf16" else 1e-4 * max(1.0, gain * gain)
    o_ref, lse_ref = O.sparse_attention(qf, kf, vf, idx_o, cnt_o, w.segment_size, w.block_size)
    out, lse = H.gpu_sparse(w, q.to(DEV), k.to(DEV), v.to(DEV),
                            torch.from_numpy(idx_o).to(DEV), torch.from_numpy(cnt_o).to(DEV))
    err = H.max_abs(out.float().cpu().numpy(), o_ref)
    print("sparse max abs err", err, "lse err", H.max_abs(lse.cpu().numpy(), lse_ref), flush=True)
    assert err <= H.TOL_OUT[dtype]
    assert H.max_abs(lse.cpu().numpy(), lse_ref) <= tol_lse
    d_ref, dlse_ref = O.dense_causal_attention(qf, kf, vf)
    dout, dlse = H.gpu_dense(w, q.to(DEV), k.to(DEV), v.to(DEV))
    err = H.max_abs(dout.float().cpu().numpy(), d_ref)
    print("dense max abs err", err, "lse err", H.max_abs(dlse.cpu().numpy(), dlse_ref), flush=True)
    assert err <= H.TOL_OUT[dtype]
    assert H.max_abs(dlse.cpu().numpy(), dlse_ref) <= tol_lse


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_full_budget_reproduces_dense_on_gpu(dtype):
    w = H.small_workload("fullbudget", 1, 2, 1, 900, 128, 32, 64, 0, dtype=dtype, unit_variance=(dtype == "bf16"))
    q, k, v = (t.to(DEV) for t in synth.make_qkv(w, threads=2))
    S = H.gpu_estimate(w, q, k)
    idx, cnt = H.gpu_select(w, q, k, S)
    o_s, lse_s = H.gpu_sparse(w, q, k, v, idx, cnt)
    o_d, lse_d = H.gpu_dense(w, q, k, v)
    # same tiles in the same order -> identical arithmetic
    assert torch.equal(o_s, o_d)
    assert torch.equal(lse_s, lse_d)


def test_degenerate_lists_and_strided_views():
    """Empty lists give zeros / -inf; a list without the diagonal leaves early rows empty; non-contiguous
    head-interleaved [B, n, H, d] storage is addressed through the strides."""
    w = H.small_workload("degenerate", 1, 2, 2, 512, 128, 32, 2, 0)
    q0, k0, v0 = synth.make_qkv(w, threads=2)
    # token-major storage: [B, n, H, d] viewed as [B, H, n, d]
    q = q0.permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)
    k = k0.permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)
    v = v0.permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)
    ll = w.list_len
    idx = np.full((1, 2, w.n_segments, ll), -1, np.int32); cnt = np.zeros((1, 2, w.n_segments), np.int32)
    idx[0, 0, 2, :2] = [0, 9]; cnt[0, 0, 2] = 2          # block 9 starts inside segment 2: partial rows
    idx[0, 1, 3, :3] = [1, 2, 15]; cnt[0, 1, 3] = 3
    o_ref, lse_ref = O.sparse_attention(synth.to_f64(q0), synth.to_f64(k0), synth.to_f64(v0), idx, cnt,
                                        w.segment_size, w.block_size)
    out = torch.full((1, w.seq_len, 2, 128), float("nan"), dtype=torch.bfloat16, device=DEV).permute(0, 2, 1, 3)
    p = H.params_for(w, q, k, out=out)
    lse = torch.full((1, 2, w.seq_len), float("nan"), dtype=torch.float32, device=DEV)
    B.critiprefill_sparse_attn(p, q, k, v, torch.from_numpy(idx).to(DEV), torch.from_numpy(cnt).to(DEV), out, lse)
    torch.cuda.synchronize()
    assert H.max_abs(out.float().cpu().numpy(), o_ref) <= 2e-2
    got = lse.cpu().numpy()
    assert np.array_equal(np.isneginf(got), np.isneginf(lse_ref))
    fin = np.isfinite(lse_ref)
    assert H.max_abs(got[fin], lse_ref[fin]) <= 2e-2
    # the same strided tensors through estimate
    S_o = O.estimate(synth.to_f64(q0), synth.to_f64(k0), w.segment_size, w.block_size)
    S_g = H.gpu_estimate(w, q, k).cpu().numpy()
    np.testing.assert_allclose(S_g, S_o, rtol=2e-4, atol=1e-30)


def test_c1_full_config():
    """BASELINE config 1 in full: fp32, 1 head, 2048 tokens, segment 128, block 32, budget 8 + diagonal."""
    w = synth.WORKLOADS["c1_fp32_2k"]
    q, k, v = synth.make_qkv(w, threads=2)
    qf, kf, vf = synth.to_f64(q), synth.to_f64(k), synth.to_f64(v)
    S = O.estimate(qf, kf, w.segment_size, w.block_size)
    Sd = O.scores_in_decision_precision(S)
    idx_o, cnt_o = O.select(Sd, w.segment_size, w.block_size, w.budget_blocks, w.local_blocks)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    S_g = H.gpu_estimate(w, qd, kd)
    np.testing.assert_allclose(S_g.cpu().numpy(), S, rtol=2e-4, atol=1e-30)
    idx_g, cnt_g = H.gpu_select(w, qd, kd, S_g)
    H.check_selection(Sd, idx_o, cnt_o, idx_g, cnt_g, w, exact=False)
    o_ref, _ = O.sparse_attention(qf, kf, vf, idx_o, cnt_o, w.segment_size, w.block_size)
    out, _ = H.gpu_sparse(w, qd, kd, vd, torch.from_numpy(idx_o).to(DEV), torch.from_numpy(cnt_o).to(DEV))
    err = H.max_abs(out.cpu().numpy(), o_ref)
    print("c1 sparse max abs err", err, flush=True)
    assert err <= 1e-4
    d_ref, _ = O.dense_causal_attention(qf, kf, vf)
    dout, _ = H.gpu_dense(w, qd, kd, vd)
    err = H.max_abs(dout.cpu().numpy(), d_ref)
    print("c1 dense max abs err", err, flush=True)
    assert err <= 1e-4


@pytest.mark.parametrize("case", [("bad_b64", 1, 2, 1, 1024, 256, 64, 3, 1, "bf16"),
                                  ("bad_b32", 1, 2, 1, 1024, 256, 32, 3, 1, "bf16"),
                                  ("bad_fp32", 1, 2, 1, 512, 128, 32, 3, 1, "fp32")], ids=lambda c: c[0])
def test_bad_device_side_lists_give_masked_rows(case):
    """A caller bug in the lists must not become an out-of-bounds access: a count beyond the list length is
    clamped, a negative count is an empty list, negative entries and entries past the last block are
    blocks without tokens.  Every access of the kernels stays inside Q/K/V and the list row for such input
    (counts are clamped to the row pitch, tokens are bounds-checked), so nothing here can fault."""
    w, q, k, v = make(case)
    print("case", case, flush=True)
    _, _, idx_o, cnt_o = oracle_lists(w, q, k)
    idx_bad, cnt_bad = idx_o.copy(), cnt_o.copy()
    idx_ref, cnt_ref = idx_o.copy(), cnt_o.copy()
    n2 = w.n_blocks
    cnt_bad[0, 0, 1] = 1_000_000                                   # A: count far beyond the row: valid prefix, then -1 padding
    idx_bad[0, 0, 2, :2] = [n2 + 5, n2 + 100]; cnt_bad[0, 0, 2] = 2   # B: blocks past the end of the sequence
    cnt_ref[0, 0, 2] = 0
    cnt_bad[0, 1, 1] = -3; cnt_ref[0, 1, 1] = 0                    # C: negative count
    idx_bad[0, 1, 2, 0] = -4; cnt_bad[0, 1, 2] = 1; cnt_ref[0, 1, 2] = 0   # D: negative entry
    idx_bad[0, 1, 3, :] = 1 << 30; cnt_bad[0, 1, 3] = 2            # E: entries whose token index overflows 32 bits
    o_ref, lse_ref = O.sparse_attention(synth.to_f64(q), synth.to_f64(k), synth.to_f64(v), idx_ref, cnt_ref,
                                        w.segment_size, w.block_size)
    out, lse = H.gpu_sparse(w, q.to(DEV), k.to(DEV), v.to(DEV),
                            torch.from_numpy(idx_bad).to(DEV), torch.from_numpy(cnt_bad).to(DEV))
    got, got_lse = out.float().cpu().numpy(), lse.cpu().numpy()
    assert np.isfinite(got).all()
    s = w.segment_size
    keep = np.ones(w.seq_len, bool); keep[3 * s:4 * s] = False     # row E of head 1: only "no fault, finite" is asked
    assert H.max_abs(got[0, 0], o_ref[0, 0]) <= H.TOL_OUT[w.dtype]
    assert H.max_abs(got[0, 1][keep], o_ref[0, 1][keep]) <= H.TOL_OUT[w.dtype]
    for (h, j) in ((0, 2), (1, 1), (1, 2)):
        assert (got[0, h, j * s:(j + 1) * s] == 0).all() and np.isneginf(got_lse[0, h, j * s:(j + 1) * s]).all()


def test_run_twice_bit_identical():
    """The whole path twice on the same inputs: every output identical bit for bit (no atomics, no
    order-dependent reductions anywhere in the kernels)."""
    case = [c for c in SMALL if c[0] == "bf16_many_segments"][0]
    w, q, k, v = make(case)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    runs = []
    for _ in range(2):
        S = H.gpu_estimate(w, qd, kd)
        idx, cnt = H.gpu_select(w, qd, kd, S)
        out, lse = H.gpu_sparse(w, qd, kd, vd, idx, cnt)
        dout, dlse = H.gpu_dense(w, qd, kd, vd)
        runs.append((S, idx, cnt, out, lse, dout, dlse))
    for a, b in zip(*runs):
        assert torch.equal(a, b)
