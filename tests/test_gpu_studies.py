"""The locality study on a small context: its figures obey what must hold for any input, and its exact per-query
sets and what it says the block lists keep are checked against the CPU checker's own per-query top-k
(Algorithm 1 + the top-k line of Algorithm 2 at segment = block = 1, which is the paper's Eq. 3)."""
import io
import json
from contextlib import redirect_stdout

import numpy as np
import pytest
import torch

from oracle import critiprefill_oracle as O
from paper_2409_12490_amd import synth

pytestmark = pytest.mark.gpu

SEQ, TOPK, HEADS = 4096, 256, (0, 31)


def oracle_sets(q, k, h, G, topk):
    """Exact sets from the checker: S at s = b = 1 is the causal softmax of q.k / sqrt(d), its top-k among the
    strictly earlier keys plus the diagonal is the list."""
    qf = synth.to_f64(q[:, h:h + 1]); kf = synth.to_f64(k[:, h // G:h // G + 1])
    S = O.estimate(qf, kf, 1, 1)
    idx, cnt = O.select(S, 1, 1, topk, 0)
    n = S.shape[-1]
    member = np.zeros((n, n), dtype=bool)
    for t in range(n):
        member[t, idx[0, 0, t, :cnt[0, 0, t]]] = True
    return member, S[0, 0]


def test_locality_study_against_the_checker():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2409_12490_amd import binding as B
    from paper_2409_12490_amd import studies
    B.load()
    buf, sets = io.StringIO(), {}
    with redirect_stdout(buf):
        studies.locality(seq_len=SEQ, heads=HEADS, topk=TOPK, keep_sets=sets)
    lines = [json.loads(x) for x in buf.getvalue().splitlines() if x.startswith("{")]
    assert len(lines) == 2
    for rec in lines:
        ov = rec["overlap_of_exact_topk_sets_by_query_distance"]
        vals = [ov[k] for k in sorted(ov, key=int)]
        assert all(0.0 <= v <= 1.0 for v in vals)
        assert vals[0] > 0.5 and vals[0] >= vals[-1]              # near queries share more than far ones
        kept, recent = rec["kept_by_block_lists"], rec["kept_by_most_recent_blocks_same_count"]
        for d in (kept, recent):
            assert 0.0 <= d["of_exact_topk_set"] <= 1.0 and 0.0 <= d["of_softmax_mass"] <= 1.0 + 1e-3
        assert kept["of_exact_topk_set"] >= recent["of_exact_topk_set"]
        assert rec["mean_listed_blocks"] <= rec["blocks_total"]

    # ---- against the checker (the same seeded inputs, drawn again on the host) ----
    w = synth.WORKLOADS["c2_llama3_8b_16k"].replace(seq_len=SEQ, name=f"llama3_8b_{SEQ // 1024}k")
    q, k, _ = synth.make_qkv(w, threads=8)
    G = w.n_q_heads // w.n_kv_heads
    n = SEQ
    rows = np.arange(n)
    full = rows >= TOPK
    for h in HEADS:
        member_o, S_o = oracle_sets(q, k, h, G, TOPK)
        print(f"head {h}: checker sets done", flush=True)
        for (label, hh), got in sets.items():
            if hh != h:
                continue
            member_g = got["member"].numpy()
            # the study ranks fp32 logits, the checker fp64 probabilities: sets may differ only where the k-th and
            # (k+1)-th key are nearly tied
            differ = int((member_g != member_o).sum())
            assert differ <= 2e-4 * member_o.sum(), (label, h, differ)
            # overlap against query distance, recomputed from the checker's sets
            size = member_o.sum(1)
            for d, v in got["overlap"].items():
                both = (member_o[:-d] & member_o[d:]).sum(1) / size[d:]
                assert abs(float(both[full[:-d]].mean()) - v) <= 2e-3, (label, h, d)
            # what the block lists of the library keep of the checker's sets, against the most recent blocks
            b, s = got["block"], got["segment"]
            n1, n2, r = n // s, n // b, s // b
            idx, cnt = got["idx"].numpy(), got["cnt"].numpy()
            listed = np.zeros((n1, n2), dtype=bool); recent = np.zeros((n1, n2), dtype=bool)
            for j in range(n1):
                listed[j, idx[j, :cnt[j]]] = True
                recent[j, (j + 1) * r - cnt[j]:(j + 1) * r] = True
            kept = {}
            for name, blocks in (("listed", listed), ("recent", recent)):
                tok_mask = blocks[rows // s][:, rows // b]
                kept[name] = float(((member_o & tok_mask).sum(1) / size)[full].mean())
            print(f"  {label}: lists keep {kept['listed']:.4f} of the checker's sets, most recent blocks {kept['recent']:.4f}", flush=True)
            assert abs(kept["listed"] - got["kept_of_set"]) <= 2e-3 and abs(kept["recent"] - got["recent_of_set"]) <= 2e-3
            assert kept["listed"] > kept["recent"]
