"""``ab_score_candidates_static`` (scoring on the library's fixed scratch array, for callers that cannot
allocate) against ``ab_score_candidates`` with a caller's workspace: the same kernels run, so scores,
choices and best scores must be equal bit for bit.  Two calls in a row share the array, the second
with a smaller input, so stale contents of the first must not leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2112_13509_amd import binding as ab
from paper_2112_13509_amd import workloads as wl
from gpu_helpers import DEV, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    ab.load()


def _both(w, S):
    """Scores / choice / best score of the first S scenarios of ``w`` from both entry points."""
    d = ab.desc_from_workload(w)
    prm = ab.Params.from_workload(w, DEV)
    dyn, scal = to_dev(w.dyn[:S]), to_dev(w.scal[:S])
    part, cred = to_dev(w.part), to_dev(w.cred)
    out = []
    for static in (False, True):
        scores = torch.full((S, w.C), float("nan"), dtype=torch.float32, device=DEV)
        idx = torch.full((S,), -7, dtype=torch.int32, device=DEV)
        best = torch.full((S,), float("nan"), dtype=torch.float32, device=DEV)
        if static:
            assert ab.ab_workspace_bytes(d, S, w.C) <= ab.ab_static_scratch_bytes()
            ab.ab_score_candidates_static(d, prm, dyn, scal, part, cred, scores, idx, best)
        else:
            ws = ab.alloc_workspace(d, S, w.C, device=DEV)
            ab.ab_score_candidates(d, prm, dyn, scal, part, cred, scores, idx, best, ws)
        torch.cuda.synchronize()
        out.append((scores.cpu().numpy(), idx.cpu().numpy(), best.cpu().numpy()))
    return out


@pytest.mark.parametrize("cfg,sizes", [(3, (24, 5)), (2, (40, 7)), (5, (48, 9))])
def test_static_scratch_equals_workspace_form(cfg, sizes):
    w = wl.make_config(cfg, S=max(sizes))
    for S in sizes:                      # the larger call first, then a smaller one on the same array
        (s0, i0, b0), (s1, i1, b1) = _both(w, S)
        assert np.isfinite(s0).all()
        assert (s0.view(np.uint32) == s1.view(np.uint32)).all(), "scores differ (cfg%d, S=%d)" % (cfg, S)
        assert (i0 == i1).all() and (i0 >= 0).all()
        assert (b0.view(np.uint32) == b1.view(np.uint32)).all()


def test_static_scratch_refuses_what_does_not_fit():
    w = wl.make_config(3, S=4)
    d = ab.desc_from_workload(w)
    prm = ab.Params.from_workload(w, DEV)
    S = 4096                                           # 2^20 candidate rows: gigabytes of activations
    assert ab.ab_workspace_bytes(d, S, w.C) > ab.ab_static_scratch_bytes()
    dyn = torch.ones(S, w.L, w.K, dtype=torch.float32, device=DEV)
    scal = torch.ones(S, len(w.scal_enc), dtype=torch.float32, device=DEV)
    idx = torch.full((S,), -7, dtype=torch.int32, device=DEV)
    rc = ab.ab_score_candidates_static(d, prm, dyn, scal, to_dev(w.part), to_dev(w.cred), None, idx, None,
                                       check=False)
    torch.cuda.synchronize()
    assert rc == -5                                    # AB_ERR_WORKSPACE, and nothing was enqueued
    assert (idx.cpu().numpy() == -7).all()
