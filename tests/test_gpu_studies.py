"""The locality study runs end to end on a small context and its figures obey what must hold for any input."""
import io
import json
from contextlib import redirect_stdout

import pytest
import torch

pytestmark = pytest.mark.gpu


def test_locality_study_small():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2409_12490_amd import binding as B
    from paper_2409_12490_amd import studies
    B.load()
    buf = io.StringIO()
    with redirect_stdout(buf):
        studies.locality(seq_len=4096, heads=(0, 31), topk=256)
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
