"""CPU checker for the CritiPrefill prefill-attention path (test infrastructure).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, float64 numpy
statement of what the path computes, written from the paper so a reader can
check it against the listings by eye.  Only the test-suite, the smoke check and
the benchmark's CPU-baseline leg may import it; the GPU library never does, and
this file imports nothing from the GPU package.

What it follows:

* ``dense_causal_attention``  – Eq. 2 (O = softmax(Q K^T / sqrt(d)) V) with the
  causal mask of an autoregressive prefill.
* ``representatives`` / ``estimate`` – Algorithm 1 "Estimation of Query
  Criticality in One Layer": reshape into segments/blocks, element-wise
  max/min representatives, four representative score matrices with a row
  softmax, S_max/S_min averages, element-wise max, block causal mask, layer
  fusion  S = alpha*S + (1-alpha)*S'.
* ``select`` – Algorithm 2 "Pruned Attention", the  argtop_k(S[j], B/block size)
  step, plus the always-kept local and diagonal blocks.
* ``sparse_attention`` – Algorithm 2, the per-segment loop: gather the listed
  blocks, softmax(Q_j K^T / sqrt(d)), times V.
* ``shared_group_scores`` / ``expand_shared_lists`` – an extension, not in the
  paper: one list per KV head from the maximum of its query heads' scores.

Readings taken where the paper is silent (each is a parameter or stated here):

* the estimation softmax uses ``score_scale`` (default 1/sqrt(d); 1.0 is the
  listing taken literally, which prints no scale);
* ``softmax_domain=0``: the row softmax runs over ALL blocks and the causal mask
  zeroes future blocks afterwards (listing order); ``1``: over visible blocks only;
* the causal mask writes 0 into blocks that lie wholly after the segment;
* the segment's own (diagonal) blocks and ``local_blocks`` blocks just before it
  are always attended, outside the budget, and a token-level causal mask
  ``u <= t`` applies inside attention;
* several heads: every query head runs the algorithms on its own, reading the
  K/V head ``h // (Hq/Hkv)``;
* ties in top-k go to the smaller block index; lists are ascending;
* a sequence length that is not a multiple of the segment or block size gives
  a shorter last segment/block (ceil division);
* ``alpha`` weighs the current layer's score, ``1-alpha`` the score handed in.

Parity pins (tests/test_oracle_pins.py): budget covering the sequence equals
dense attention; segment = block = 1 equals per-query top-k (Eq. 3); softmax
rows sum to one; dense attention against a library routine; brute-force token
masks on tiny inputs; closed forms (constant V, equal keys, hand-worked
softmax of log-integers); planted block; invariances; nesting in the budget.
No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

NEG_INF = -np.inf


def _softmax_lastaxis(z: np.ndarray) -> np.ndarray:
    m = np.max(z, axis=-1, keepdims=True)
    e = np.exp(z - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def _kv_head(h: int, n_q_heads: int, n_kv_heads: int) -> int:
    return h // (n_q_heads // n_kv_heads)


# --------------------------------------------------------------------------
# Eq. 2: dense causal attention
# --------------------------------------------------------------------------
def dense_causal_attention(q, k, v, attn_scale=None, row_chunk=256, rows=None):
    """Eq. 2 with the causal mask: O[t] = sum_{u<=t} softmax_u(q_t.k_u/sqrt(d)) v_u.

    q: [B,Hq,n,d]; k, v: [B,Hkv,n,d] (float64).  ``rows``: optional 1-D array of
    query positions; then only those rows are returned, shape [B,Hq,len(rows),d].
    Returns (O, LSE) with LSE = log sum_u exp(scaled logit) (natural log).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, Hq, n, d = q.shape
    Hkv = k.shape[1]
    scale = 1.0 / np.sqrt(d) if attn_scale is None else float(attn_scale)
    pos = np.arange(n) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.zeros((B, Hq, len(pos), d))
    lse = np.zeros((B, Hq, len(pos)))
    for b in range(B):
        for h in range(Hq):
            kh, vh = k[b, _kv_head(h, Hq, Hkv)], v[b, _kv_head(h, Hq, Hkv)]
            for c0 in range(0, len(pos), row_chunk):
                t = pos[c0:c0 + row_chunk]
                hi = int(t.max()) + 1
                z = scale * (q[b, h, t] @ kh[:hi].T)
                z[np.arange(hi)[None, :] > t[:, None]] = NEG_INF
                m = z.max(axis=1, keepdims=True)
                e = np.exp(z - m)
                l = e.sum(axis=1, keepdims=True)
                out[b, h, c0:c0 + len(t)] = (e / l) @ vh[:hi]
                lse[b, h, c0:c0 + len(t)] = (m + np.log(l))[:, 0]
    return out, lse


# --------------------------------------------------------------------------
# Algorithm 1: criticality estimation
# --------------------------------------------------------------------------
def _group_max_min(x: np.ndarray, size: int):
    """Element-wise max and min over consecutive groups of ``size`` rows of x [n,d]."""
    n, d = x.shape
    groups = -(-n // size)
    hi = np.empty((groups, d))
    lo = np.empty((groups, d))
    for g in range(groups):
        rows = x[g * size:min(n, (g + 1) * size)]
        hi[g] = rows.max(axis=0)
        lo[g] = rows.min(axis=0)
    return hi, lo


def representatives(q, k, segment_size, block_size):
    """Algorithm 1, the reshape and max/min lines: Q_max,Q_min [B,Hq,n1,d], K_max,K_min [B,Hkv,n2,d]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    B, Hq, n, d = q.shape
    Hkv = k.shape[1]
    n1, n2 = -(-n // segment_size), -(-n // block_size)
    qmax = np.empty((B, Hq, n1, d)); qmin = np.empty((B, Hq, n1, d))
    kmax = np.empty((B, Hkv, n2, d)); kmin = np.empty((B, Hkv, n2, d))
    for b in range(B):
        for h in range(Hq):
            qmax[b, h], qmin[b, h] = _group_max_min(q[b, h], segment_size)
        for h in range(Hkv):
            kmax[b, h], kmin[b, h] = _group_max_min(k[b, h], block_size)
    return qmax, qmin, kmax, kmin


def four_softmaxes(qmax, qmin, kmax, kmin, r, score_scale, softmax_domain=0):
    """Algorithm 1, S_1..S_4 for one head: softmax over blocks of the four
    representative products (max.max, max.min, min.max, min.min), in that order.

    ``r`` = blocks per segment.  Domain 0: softmax over every block.  Domain 1:
    over the visible blocks i < (j+1)*r only (the others get probability 0).
    """
    n1, n2 = qmax.shape[0], kmax.shape[0]
    outs = []
    for qa, kb in ((qmax, kmax), (qmax, kmin), (qmin, kmax), (qmin, kmin)):
        z = score_scale * (qa @ kb.T)
        if softmax_domain == 0:
            outs.append(_softmax_lastaxis(z))
        else:
            s = np.zeros((n1, n2))
            for j in range(n1):
                vis = min(n2, (j + 1) * r)
                s[j, :vis] = _softmax_lastaxis(z[j, :vis])
            outs.append(s)
    return outs


def estimate(q, k, segment_size, block_size, score_scale=None, softmax_domain=0,
             prev_scores=None, alpha=1.0):
    """Algorithm 1: criticality score S [B,Hq,n1,n2] (float64, probability domain).

    ``prev_scores`` is S' of the previous layer (the fused score that layer
    returned); when it is None the fusion line is skipped.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    B, Hq, n, d = q.shape
    Hkv = k.shape[1]
    if segment_size % block_size:
        raise ValueError("block size must divide segment size")
    r = segment_size // block_size
    scale = 1.0 / np.sqrt(d) if score_scale is None else float(score_scale)
    qmax, qmin, kmax, kmin = representatives(q, k, segment_size, block_size)
    n1, n2 = qmax.shape[2], kmax.shape[2]
    S = np.empty((B, Hq, n1, n2))
    block = np.arange(n2)[None, :]
    first_future = (np.arange(n1)[:, None] + 1) * r
    for b in range(B):
        for h in range(Hq):
            g = _kv_head(h, Hq, Hkv)
            s1, s2, s3, s4 = four_softmaxes(qmax[b, h], qmin[b, h], kmax[b, g], kmin[b, g],
                                            r, scale, softmax_domain)
            s_max = (s1 + s3) / 2.0
            s_min = (s2 + s4) / 2.0
            s = np.maximum(s_max, s_min)
            s[block >= first_future] = 0.0                      # causal mask on blocks
            if prev_scores is not None:
                s = alpha * s + (1.0 - alpha) * np.asarray(prev_scores, dtype=np.float64)[b, h]
            S[b, h] = s
    return S


def scores_in_decision_precision(scores):
    """Round S to the precision the top-k decision is taken in: float32 (the type
    of the score buffer at the library boundary) with subnormals flushed to zero."""
    s32 = np.asarray(scores, dtype=np.float64).astype(np.float32)
    s32[np.abs(s32) < np.finfo(np.float32).tiny] = 0.0
    return s32


# --------------------------------------------------------------------------
# Algorithm 2: selection and pruned attention
# --------------------------------------------------------------------------
def select(scores, segment_size, block_size, budget_blocks, local_blocks=0):
    """Block list per segment: top-``budget_blocks`` of S[j] among the candidate
    blocks (those before the local window), then the local blocks, then the
    segment's own blocks.  Ascending; ties go to the smaller block index.

    scores: [B,H,n1,n2] in the precision the decision is to be taken in.
    Returns idx int32 [B,H,n1,Lmax] (unused tail -1) and cnt int32 [B,H,n1].
    """
    scores = np.asarray(scores)
    B, H, n1, n2 = scores.shape
    r = segment_size // block_size
    lmax = budget_blocks + local_blocks + r
    idx = np.full((B, H, n1, lmax), -1, dtype=np.int32)
    cnt = np.zeros((B, H, n1), dtype=np.int32)
    for b in range(B):
        for h in range(H):
            for j in range(n1):
                diag_lo = j * r
                diag_hi = min(n2, (j + 1) * r)
                n_local = min(local_blocks, diag_lo)
                n_cand = diag_lo - n_local
                kj = min(budget_blocks, n_cand)
                row = scores[b, h, j, :n_cand]
                # stable sort of -score: equal scores keep ascending index order
                order = np.argsort(-row, kind="stable")[:kj]
                lst = np.concatenate([np.sort(order), np.arange(n_cand, diag_hi)])
                idx[b, h, j, :len(lst)] = lst
                cnt[b, h, j] = len(lst)
    return idx, cnt


def shared_group_scores(scores, n_kv_heads):
    """Extension beyond the paper (which describes one head and gives no rule for sharing a list between
    heads): the score a KV head's shared list is chosen from is the element-wise maximum of S over the
    query heads that read that KV head.  scores [B,Hq,n1,n2] -> [B,Hkv,n1,n2].  ``select`` on the result
    gives one list per (batch, KV head, segment); ``expand_shared_lists`` hands it to every query head."""
    scores = np.asarray(scores)
    B, Hq, n1, n2 = scores.shape
    G = Hq // n_kv_heads
    out = np.empty((B, n_kv_heads, n1, n2), dtype=scores.dtype)
    for g in range(n_kv_heads):
        members = [h for h in range(Hq) if _kv_head(h, Hq, n_kv_heads) == g]
        assert len(members) == G
        out[:, g] = scores[:, members].max(axis=1)
    return out


def expand_shared_lists(block_idx, block_cnt, n_q_heads):
    """Per-KV-head lists [B,Hkv,n1,L] / [B,Hkv,n1] repeated for every query head of the group."""
    Hkv = block_idx.shape[1]
    heads = [_kv_head(h, n_q_heads, Hkv) for h in range(n_q_heads)]
    return block_idx[:, heads].copy(), block_cnt[:, heads].copy()


def sparse_attention(q, k, v, block_idx, block_cnt, segment_size, block_size,
                     attn_scale=None, segments=None, return_probs=False):
    """Algorithm 2 loop: for each segment gather the listed K/V blocks and attend.

    Token-level causality (key position <= query position) is enforced inside
    the listed blocks.  A query with no visible key gets output 0 and LSE -inf.
    ``segments``: optional iterable of (b, h, j) triples; only those segments are
    computed and everything else in the returned arrays stays 0.
    Returns (O [B,Hq,n,d], LSE [B,Hq,n]) and, if ``return_probs``, a dict
    (b,h,j) -> (key positions, probability matrix [rows, keys]).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, Hq, n, d = q.shape
    Hkv = k.shape[1]
    n1 = -(-n // segment_size)
    scale = 1.0 / np.sqrt(d) if attn_scale is None else float(attn_scale)
    out = np.zeros((B, Hq, n, d))
    lse = np.zeros((B, Hq, n))
    probs = {}
    todo = segments if segments is not None else [(b, h, j) for b in range(B) for h in range(Hq) for j in range(n1)]
    for (b, h, j) in todo:
        g = _kv_head(h, Hq, Hkv)
        blocks = block_idx[b, h, j, :block_cnt[b, h, j]]
        if len(blocks):
            u = np.concatenate([np.arange(i * block_size, min(n, (i + 1) * block_size)) for i in blocks])
        else:
            u = np.zeros(0, dtype=np.int64)
        t = np.arange(j * segment_size, min(n, (j + 1) * segment_size))
        z = scale * (q[b, h, t] @ k[b, g, u].T)
        z[u[None, :] > t[:, None]] = NEG_INF
        m = z.max(axis=1, keepdims=True) if len(u) else np.full((len(t), 1), NEG_INF)
        dead = ~np.isfinite(m[:, 0])
        m_safe = np.where(np.isfinite(m), m, 0.0)
        e = np.exp(z - m_safe)
        l = e.sum(axis=1, keepdims=True)
        l_safe = np.where(l > 0, l, 1.0)
        p = e / l_safe
        o = p @ v[b, g, u]
        o[dead] = 0.0
        out[b, h, t] = o
        with np.errstate(divide="ignore"):
            lse[b, h, t] = np.where(dead, NEG_INF, (m_safe + np.log(l_safe))[:, 0])
        if return_probs:
            probs[(b, h, j)] = (u, p)
    if return_probs:
        return out, lse, probs
    return out, lse

