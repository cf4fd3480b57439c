"""pruner_topk_static (selection with the scratch inside the library, for callers that cannot allocate) against
pruner_topk: same index lists and values, on two calls in a row that share the library's scratch, the second on a smaller
input, on both selection routes."""
import numpy as np
import pytest

import paper_2402_02361_amd as P

pytestmark = pytest.mark.gpu


def _scores(n, seed, ties):
    rng = np.random.default_rng(seed)
    s = -np.exp(rng.normal(size=n)).astype(np.float32)
    if ties:
        s = np.round(s, 1)            # many equal scores: the index tie-break decides
    return s


@pytest.mark.parametrize("lens_big, lens_small, k", [
    ([300000, 150001, 70000], [40000, 90003], 512),     # large route twice
    ([200000, 9000], [5000, 4100, 7777], 4096),         # large route, then the one-workgroup route
    ([3000] * 16, [257], 64),                           # the limit of 16 segments, then one short segment
])
def test_static_scratch_selection_equals_pruner_topk(lens_big, lens_small, k):
    import torch
    for ties in (False, True):
        for call, lens in enumerate((lens_big, lens_small)):
            seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
            n, n_sg = int(seg[-1]), len(lens)
            score = torch.from_numpy(_scores(n, 11 + call, ties)).cuda()
            idx = torch.full((n_sg, k), -1, dtype=torch.int32, device="cuda")
            val = torch.full((n_sg, k), float("nan"), dtype=torch.float32, device="cuda")
            print(f"pruner_topk_static: call {call}, segments {lens}, k {k}, ties {ties}", flush=True)
            P.topk_static(score, seg, k, idx, val)
            want_idx, want_val = P.topk(score, seg, k)
            torch.cuda.synchronize()
            assert torch.equal(idx, want_idx)
            assert torch.equal(val.view(torch.int32), want_val.view(torch.int32))


def test_static_scratch_refuses_more_segments_than_it_holds():
    import torch
    seg = np.arange(18, dtype=np.int64) * 100
    score = torch.zeros(1700, device="cuda")
    idx = torch.empty((17, 10), dtype=torch.int32, device="cuda")
    with pytest.raises(P.PrunerError):
        P.topk_static(score, seg, 10, idx)
