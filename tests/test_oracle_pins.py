"""Pins for the CPU checker: closed forms, library routines, brute force, invariants.

Each test is chosen so that a plausible slip in oracle/critiprefill_oracle.py (a
dropped term, a wrong index, a transposed operand, a missing mask) fails it.
All run on the CPU.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import critiprefill_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_qkv(seed, B, Hq, Hkv, n, d, walk=True):
    g = np.random.default_rng(seed)
    def one(H):
        x = g.standard_normal((B, H, n, d))
        if walk:
            x = x + np.cumsum(0.3 * g.standard_normal((B, H, n, d)), axis=2)
        return x
    return one(Hq), one(Hkv), one(Hkv)


# ---- Eq. 2 against a library routine and a ten-line numpy statement ---------------
def numpy_masked_attention(q, k, v, mask, scale):
    """softmax(mask(q k^T * scale)) v for one head; mask[t,u] True = visible."""
    z = scale * q @ k.T
    z = np.where(mask, z, -np.inf)
    z = z - z.max(axis=1, keepdims=True)
    p = np.exp(z)
    p /= p.sum(axis=1, keepdims=True)
    return p @ v, p


@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (4, 2), (6, 1)])
def test_dense_matches_torch_sdpa_and_numpy(Hq, Hkv):
    B, n, d = 2, 67, 16
    q, k, v = rand_qkv(1, B, Hq, Hkv, n, d)
    o, lse = O.dense_causal_attention(q, k, v)
    G = Hq // Hkv
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq, tk.repeat_interleave(G, dim=1), tv.repeat_interleave(G, dim=1), is_causal=True).numpy()
    np.testing.assert_allclose(o, ref, rtol=1e-11, atol=1e-12)
    tril = np.tril(np.ones((n, n), dtype=bool))
    for b, h in itertools.product(range(B), range(Hq)):
        ref2, p = numpy_masked_attention(q[b, h], k[b, h // G], v[b, h // G], tril, 1 / np.sqrt(d))
        np.testing.assert_allclose(o[b, h], ref2, rtol=1e-11, atol=1e-12)
        z = (q[b, h] @ k[b, h // G].T) / np.sqrt(d)
        ref_lse = np.array([np.log(np.exp(z[t, :t + 1]).sum()) for t in range(n)])
        np.testing.assert_allclose(lse[b, h], ref_lse, rtol=1e-11)


def test_dense_row_subset_and_scale():
    q, k, v = rand_qkv(2, 1, 2, 1, 50, 8)
    full, lse = O.dense_causal_attention(q, k, v, attn_scale=0.37)
    rows = np.array([0, 7, 49, 13])
    part, lse_p = O.dense_causal_attention(q, k, v, attn_scale=0.37, rows=rows)
    np.testing.assert_allclose(part, full[:, :, rows], rtol=1e-12)
    np.testing.assert_allclose(lse_p, lse[:, :, rows], rtol=1e-12)
    tril = np.tril(np.ones((50, 50), dtype=bool))
    ref, _ = numpy_masked_attention(q[0, 1], k[0, 0], v[0, 0], tril, 0.37)
    np.testing.assert_allclose(full[0, 1], ref, rtol=1e-11)


# ---- P1: a budget that covers the sequence reproduces dense attention ---------------
@pytest.mark.parametrize("n,s,b,L", [(96, 32, 8, 0), (100, 32, 8, 1), (61, 16, 16, 2), (64, 8, 4, 0)])
def test_full_budget_equals_dense(n, s, b, L):
    q, k, v = rand_qkv(3, 1, 4, 2, n, 8)
    S = O.estimate(q, k, s, b)
    n2 = -(-n // b)
    idx, cnt = O.select(S, s, b, budget_blocks=n2, local_blocks=L)
    r = s // b
    for j in range(idx.shape[2]):
        want = np.arange(min(n2, (j + 1) * r))
        assert cnt[0, 0, j] == len(want)
        np.testing.assert_array_equal(idx[0, 0, j, :len(want)], want)
        assert (idx[0, 0, j, len(want):] == -1).all()
    o_s, lse_s = O.sparse_attention(q, k, v, idx, cnt, s, b)
    o_d, lse_d = O.dense_causal_attention(q, k, v)
    np.testing.assert_allclose(o_s, o_d, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(lse_s, lse_d, rtol=1e-11)


# ---- P2: segment = block = 1 is exact per-query top-k (Eq. 3) -----------------------
@pytest.mark.parametrize("kbud", [1, 3, 7])
def test_unit_segments_reduce_to_per_query_topk(kbud):
    n, d = 40, 8
    q, k, v = rand_qkv(4, 1, 2, 1, n, d, walk=False)
    S = O.estimate(q, k, 1, 1)
    for h in range(2):
        z = (q[0, h] @ k[0, 0].T) / np.sqrt(d)
        # with max = min representatives the four softmaxes coincide -> S is the masked softmax
        full = np.exp(z - z.max(1, keepdims=True)); full /= full.sum(1, keepdims=True)
        np.testing.assert_allclose(S[0, h], np.tril(full), rtol=1e-11, atol=1e-300)
    idx, cnt = O.select(S, 1, 1, kbud, 0)
    for h in range(2):
        raw = q[0, h] @ k[0, 0].T                         # Eq. 3 ranks q_i K^T (softmax is monotone)
        for t in range(n):
            top = np.sort(np.argsort(-raw[t, :t], kind="stable")[:kbud])
            want = np.concatenate([top, [t]])
            assert cnt[0, h, t] == len(want)
            np.testing.assert_array_equal(idx[0, h, t, :len(want)], want)
    # attention over that list = exact attention over the top-k keys plus the query's own key
    o, _ = O.sparse_attention(q, k, v, idx, cnt, 1, 1)
    for h in range(2):
        for t in range(n):
            keys = idx[0, h, t, :cnt[0, h, t]]
            z = (k[0, 0, keys] @ q[0, h, t]) / np.sqrt(d)
            p = np.exp(z - z.max()); p /= p.sum()
            np.testing.assert_allclose(o[0, h, t], p @ v[0, 0, keys], rtol=1e-11, atol=1e-13)


# ---- P3: softmax rows sum to one, ranges -------------------------------------------
@pytest.mark.parametrize("domain", [0, 1])
def test_softmax_rows_sum_to_one(domain):
    n, s, b, d = 128, 32, 8, 16
    q, k, v = rand_qkv(5, 1, 2, 2, n, d)
    qmax, qmin, kmax, kmin = O.representatives(q, k, s, b)
    r = s // b
    four = O.four_softmaxes(qmax[0, 1], qmin[0, 1], kmax[0, 1], kmin[0, 1], r, 1 / np.sqrt(d), domain)
    for sm in four:
        assert (sm >= 0).all() and (sm <= 1).all()
        np.testing.assert_allclose(sm.sum(axis=1), 1.0, rtol=1e-12)
        if domain == 1:
            for j in range(sm.shape[0]):
                assert (sm[j, (j + 1) * r:] == 0).all()
    S = O.estimate(q, k, s, b, softmax_domain=domain)
    assert (S >= 0).all() and (S <= 1).all()
    if domain == 1:            # max of two distributions over the same visible support
        rs = S[0, 1].sum(axis=1)
        assert (rs >= 1 - 1e-12).all() and (rs <= 2 + 1e-12).all()
    # attention probabilities of every query sum to one
    idx, cnt = O.select(S, s, b, 3, 1)
    _, _, probs = O.sparse_attention(q, k, v, idx, cnt, s, b, return_probs=True)
    for (_, p) in probs.values():
        np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-12)


# ---- P5: brute force with explicit token masks on tiny inputs ----------------------
def brute_token_mask(n, s, b, blocks, j):
    mask = np.zeros((n, n), dtype=bool)
    for t in range(j * s, min(n, (j + 1) * s)):
        for i in blocks:
            for u in range(i * b, min(n, (i + 1) * b)):
                if u <= t:
                    mask[t, u] = True
    return mask


@pytest.mark.parametrize("n,s,b,kb,L,Hq,Hkv", [(64, 16, 4, 2, 1, 4, 2), (50, 16, 8, 1, 0, 2, 1), (37, 8, 2, 3, 2, 3, 3)])
def test_sparse_matches_bruteforce_mask(n, s, b, kb, L, Hq, Hkv):
    d = 8
    q, k, v = rand_qkv(6, 2, Hq, Hkv, n, d)
    S = O.estimate(q, k, s, b)
    idx, cnt = O.select(S, s, b, kb, L)
    o, _ = O.sparse_attention(q, k, v, idx, cnt, s, b)
    G = Hq // Hkv
    n1 = -(-n // s)
    for bb, h in itertools.product(range(2), range(Hq)):
        mask = np.zeros((n, n), dtype=bool)
        for j in range(n1):
            mask |= brute_token_mask(n, s, b, idx[bb, h, j, :cnt[bb, h, j]], j)
        assert mask.diagonal().all()                      # every query sees itself
        ref, _ = numpy_masked_attention(q[bb, h], k[bb, h // G], v[bb, h // G], mask, 1 / np.sqrt(d))
        np.testing.assert_allclose(o[bb, h], ref, rtol=1e-11, atol=1e-13)


def brute_estimate_one(qh, kh, s, b, scale, domain):
    """Token-level loops, scalar arithmetic, for tiny inputs."""
    n, d = qh.shape
    n1, n2, r = -(-n // s), -(-n // b), s // b
    S = np.zeros((n1, n2))
    for j in range(n1):
        qs = qh[j * s:(j + 1) * s]
        reps_q = [qs.max(0), qs.min(0)]
        cols = n2 if domain == 0 else min(n2, (j + 1) * r)
        sm = {}
        for a in range(2):
            for c in range(2):
                z = []
                for i in range(cols):
                    ks = kh[i * b:(i + 1) * b]
                    rep_k = ks.max(0) if c == 0 else ks.min(0)
                    z.append(scale * sum(reps_q[a][e] * rep_k[e] for e in range(d)))
                z = np.array(z); e = np.exp(z - z.max()); sm[(a, c)] = e / e.sum()
        smax = (sm[(0, 0)] + sm[(1, 0)]) / 2
        smin = (sm[(0, 1)] + sm[(1, 1)]) / 2
        val = np.maximum(smax, smin)
        for i in range(cols):
            if i < (j + 1) * r:
                S[j, i] = val[i]
    return S


@pytest.mark.parametrize("domain", [0, 1])
@pytest.mark.parametrize("n,s,b", [(48, 16, 4), (45, 16, 8), (20, 4, 4)])
def test_estimate_matches_token_level_loops(domain, n, s, b):
    d = 6
    q, k, _ = rand_qkv(7, 1, 4, 2, n, d)
    S = O.estimate(q, k, s, b, score_scale=0.5, softmax_domain=domain)
    for h in range(4):
        ref = brute_estimate_one(q[0, h], k[0, h // 2], s, b, 0.5, domain)
        np.testing.assert_allclose(S[0, h], ref, rtol=1e-11, atol=1e-300)


# ---- P6: closed forms -------------------------------------------------------------
@pytest.mark.parametrize("fixture,block", [("alg1_log_integer_scores.txt", 1), ("alg1_maxmin_pairing.txt", 2)])
def test_golden_hand_worked_scores(fixture, block):
    rows = {}
    with open(os.path.join(GOLDEN, fixture)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            parts = line.split()
            rows[int(parts[0])] = [float(Fraction(x)) for x in parts[1:]]
    q = np.array([1.0, 1.0, 2.0, 1.0]).reshape(1, 1, 4, 1)
    k = np.array([0.0, np.log(2.0), np.log(3.0), 0.0]).reshape(1, 1, 4, 1)
    S = O.estimate(q, k, 2, block, score_scale=1.0)
    for j, want in rows.items():
        np.testing.assert_allclose(S[0, 0, j], want, rtol=1e-12, atol=1e-15)


def test_constant_values_give_constant_output():
    n, s, b, d = 96, 32, 8, 8
    q, k, v = rand_qkv(8, 1, 2, 1, n, d)
    c = np.arange(1, d + 1, dtype=np.float64)
    v[:] = c
    S = O.estimate(q, k, s, b)
    idx, cnt = O.select(S, s, b, 2, 1)
    o, _ = O.sparse_attention(q, k, v, idx, cnt, s, b)
    np.testing.assert_allclose(o, np.broadcast_to(c, o.shape), rtol=1e-12)
    o, _ = O.dense_causal_attention(q, k, v)
    np.testing.assert_allclose(o, np.broadcast_to(c, o.shape), rtol=1e-12)


def test_equal_keys_give_uniform_weights_and_mean_position():
    n, s, b, d = 80, 16, 4, 4
    q, k, v = rand_qkv(9, 1, 1, 1, n, d)
    k[:] = k[0, 0, 0]
    v[0, 0, :, :] = np.arange(n)[:, None]
    r = s // b
    n2 = n // b
    for domain in (0, 1):
        S = O.estimate(q, k, s, b, softmax_domain=domain)
        for j in range(n // s):
            vis = (j + 1) * r
            want = 1.0 / (n2 if domain == 0 else vis)
            np.testing.assert_allclose(S[0, 0, j, :vis], want, rtol=1e-12)
            assert (S[0, 0, j, vis:] == 0).all()
    S = O.estimate(q, k, s, b)
    idx, cnt = O.select(S, s, b, 2, 1)
    # all candidates tie -> the two smallest indices win
    for j in range(n // s):
        n_cand = max(0, j * r - 1)
        assert list(idx[0, 0, j, :min(2, n_cand)]) == list(range(min(2, n_cand)))
    o, lse = O.sparse_attention(q, k, v, idx, cnt, s, b)
    for t in range(n):
        j = t // s
        seen = [u for i in idx[0, 0, j, :cnt[0, 0, j]] for u in range(i * b, (i + 1) * b) if u <= t]
        np.testing.assert_allclose(o[0, 0, t], np.mean(seen), rtol=1e-12)
        z = (q[0, 0, t] @ k[0, 0, 0]) / np.sqrt(d)
        np.testing.assert_allclose(lse[0, 0, t], z + np.log(len(seen)), rtol=1e-12)


# ---- P7: a planted block must be selected -------------------------------------------
def test_planted_block_is_selected():
    n, s, b, d = 256, 32, 8, 16
    q, k, v = rand_qkv(10, 1, 1, 1, n, d, walk=False)
    j, target = 6, 5                                     # segment 6 starts at block 24
    qmax = q[0, 0, j * s:(j + 1) * s].max(0)
    k[0, 0, target * b:(target + 1) * b] += 4.0 * qmax / np.linalg.norm(qmax) * np.sqrt(d)
    S = O.estimate(q, k, s, b)
    cand = S[0, 0, j, :j * (s // b)]
    assert np.argmax(cand) == target
    idx, cnt = O.select(S, s, b, 1, 0)
    assert idx[0, 0, j, 0] == target


# ---- P8: invariances --------------------------------------------------------------
def test_invariances():
    n, s, b, d = 96, 32, 8, 8
    q, k, v = rand_qkv(11, 1, 2, 1, n, d)
    S = O.estimate(q, k, s, b)
    idx, cnt = O.select(S, s, b, 2, 0)
    o, _ = O.sparse_attention(q, k, v, idx, cnt, s, b)
    g = np.random.default_rng(0)
    # permuting tokens inside a strictly-past block (K and V together)
    k2, v2 = k.copy(), v.copy()
    perm = g.permutation(b)
    k2[0, 0, 0:b] = k[0, 0, 0:b][perm]; v2[0, 0, 0:b] = v[0, 0, 0:b][perm]
    S2 = O.estimate(q, k2, s, b)
    np.testing.assert_allclose(S2, S, rtol=1e-12, atol=1e-300)
    o2, _ = O.sparse_attention(q, k2, v2, idx, cnt, s, b)
    np.testing.assert_allclose(o2[0, :, s:], o[0, :, s:], rtol=1e-11, atol=1e-13)   # segments after block 0's own
    # permuting queries inside a segment leaves S unchanged
    q2 = q.copy(); perm = g.permutation(s)
    q2[0, :, s:2 * s] = q[0, :, s:2 * s][:, perm]
    np.testing.assert_allclose(O.estimate(q2, k, s, b), S, rtol=1e-12, atol=1e-300)
    # V scaling
    o3, _ = O.sparse_attention(q, k, 2.5 * v, idx, cnt, s, b)
    np.testing.assert_allclose(o3, 2.5 * o, rtol=1e-12)
    # layer fusion end points and midpoint
    prev = g.random(S.shape)
    np.testing.assert_allclose(O.estimate(q, k, s, b, prev_scores=prev, alpha=1.0), S, rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(O.estimate(q, k, s, b, prev_scores=prev, alpha=0.0), prev, rtol=1e-12)
    np.testing.assert_allclose(O.estimate(q, k, s, b, prev_scores=prev, alpha=0.25), 0.25 * S + 0.75 * prev, rtol=1e-12)


def test_gqa_head_mapping():
    n, s, b, d = 64, 16, 4, 8
    q, k, v = rand_qkv(12, 1, 4, 2, n, d)
    S = O.estimate(q, k, s, b)
    idx, cnt = O.select(S, s, b, 2, 1)
    o, _ = O.sparse_attention(q, k, v, idx, cnt, s, b)
    for h in range(4):
        g = h // 2
        S1 = O.estimate(q[:, h:h + 1], k[:, g:g + 1], s, b)
        np.testing.assert_allclose(S1[0, 0], S[0, h], rtol=1e-12, atol=1e-300)
        o1, _ = O.sparse_attention(q[:, h:h + 1], k[:, g:g + 1], v[:, g:g + 1], idx[:, h:h + 1], cnt[:, h:h + 1], s, b)
        np.testing.assert_allclose(o1[0, 0], o[0, h], rtol=1e-12, atol=1e-300)


# ---- P9: nesting in the budget, error goes to zero ----------------------------------
def test_lists_nest_in_budget_and_error_vanishes():
    n, s, b, d = 256, 32, 8, 8
    q, k, v = rand_qkv(13, 1, 2, 2, n, d)
    S = O.estimate(q, k, s, b)
    dense, _ = O.dense_causal_attention(q, k, v)
    prev_sets, errs = None, []
    for kb in [0, 1, 2, 4, 8, 16, 32]:
        idx, cnt = O.select(S, s, b, kb, 0)
        sets = [[set(idx[0, h, j, :cnt[0, h, j]]) for j in range(n // s)] for h in range(2)]
        if prev_sets is not None:
            for h in range(2):
                for j in range(n // s):
                    assert prev_sets[h][j] <= sets[h][j]
        prev_sets = sets
        o, _ = O.sparse_attention(q, k, v, idx, cnt, s, b)
        errs.append(np.abs(o - dense).max())
    assert errs[-1] < 1e-12 and errs[0] > 1e-3


# ---- select: structure, ties, ragged ------------------------------------------------
def test_select_structure_and_ties():
    s, b, kb, L = 8, 2, 3, 1
    r = s // b
    n1, n2 = 5, 19                                       # ragged: 37 tokens -> last block index 18
    g = np.random.default_rng(3)
    S = g.random((1, 1, n1, n2)).astype(np.float32)
    S[0, 0, 3, :] = 0.5                                  # full tie in row 3
    S[0, 0, 4, 2] = S[0, 0, 4, 9] = 2.0                  # two clear winners
    S[0, 0, 4, [0, 5, 7]] = 1.5                          # three-way tie for the last slot
    idx, cnt = O.select(S, s, b, kb, L)
    assert idx.shape == (1, 1, n1, kb + L + r)
    assert cnt[0, 0, 0] == r and list(idx[0, 0, 0, :r]) == [0, 1, 2, 3]
    assert list(idx[0, 0, 3, :cnt[0, 0, 3]]) == [0, 1, 2, 11, 12, 13, 14, 15]
    assert list(idx[0, 0, 4, :cnt[0, 0, 4]]) == [0, 2, 9, 15, 16, 17, 18]
    for j in range(n1):
        row = idx[0, 0, j, :cnt[0, 0, j]]
        assert (np.diff(row) > 0).all()
        assert (idx[0, 0, j, cnt[0, 0, j]:] == -1).all()


def test_decision_precision_flushes_subnormals():
    x = np.array([1e-50, 1e-40, 2e-38, 0.5])
    y = O.scores_in_decision_precision(x)
    assert y.dtype == np.float32
    assert y[0] == 0 and y[1] == 0 and y[2] > 0 and y[3] == np.float32(0.5)


def test_shared_group_scores_bruteforce_and_special_cases():
    """The shared-list extension: element by element against python loops; one head per group is the
    identity; a list chosen from the group maximum contains each member head's single best candidate."""
    rng = np.random.default_rng(5)
    B_, Hq, Hkv, n1, n2, r = 2, 6, 2, 5, 20, 4
    S = rng.random((B_, Hq, n1, n2)).astype(np.float32)
    Sg = O.shared_group_scores(S, Hkv)
    G = Hq // Hkv
    for b in range(B_):
        for g in range(Hkv):
            for j in range(n1):
                for i in range(n2):
                    assert Sg[b, g, j, i] == max(S[b, g * G + m, j, i] for m in range(G))
    np.testing.assert_array_equal(O.shared_group_scores(S, Hq), S)
    idx_g, cnt_g = O.select(Sg, r * 2, 2, 3, 0)
    idx_h, cnt_h = O.expand_shared_lists(idx_g, cnt_g, Hq)
    assert idx_h.shape[1] == Hq
    for b in range(B_):
        for h in range(Hq):
            np.testing.assert_array_equal(idx_h[b, h], idx_g[b, h // G])
            for j in range(1, n1):
                n_cand = j * r
                best = int(np.argmax(S[b, h, j, :n_cand]))
                shared = idx_g[b, h // G, j, :cnt_g[b, h // G, j]]
                # the head's best block is in the shared list unless 3 blocks of the group beat it
                beaten_by = int((Sg[b, h // G, j, :n_cand] > S[b, h, j, best]).sum())
                assert best in shared or beaten_by >= 3
