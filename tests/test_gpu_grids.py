"""Per-scenario candidate grids (every scenario brings its own partition sizes and credit multiples) on the GPU
against the oracle, on every scoring path: the single-launch path, one hidden layer, the generic tiles in fp32
and bf16, and the 256 x 256 kernels (streaming and one tile per work-group)."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2112_13509_amd import binding as ab
from paper_2112_13509_amd import workloads as wl
from helpers import oracle_model
from gpu_helpers import to_dev, DEV, check_scores, matched_scores

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    ab.load()


def draw_grids(S, P, Q, seed):
    rng = np.random.default_rng(seed)
    part = np.sort(np.exp(rng.uniform(np.log(16e3), np.log(64e6), size=(S, P))), axis=1).astype(np.float32)
    cred = np.sort(rng.uniform(1.0, 16.0, size=(S, Q)), axis=1).astype(np.float32)
    return part, cred


@pytest.mark.parametrize("dtype,hidden,S,P,Q,what", [
    ("f32", [64, 64], 3, 8, 8, "single launch"),
    ("bf16", [64, 64], 2, 4, 8, "single launch, bf16"),
    ("f32", [128], 37, 5, 7, "one hidden layer"),
    ("f32", [256, 64], 41, 9, 7, "generic tiles, fp32, ragged"),
    ("bf16", [192, 128, 64], 300, 8, 8, "generic tiles, bf16"),
    ("bf16", [256, 256, 256], 70, 16, 16, "256 x 256 streaming kernels"),
    ("bf16", [64, 256, 256], 70, 16, 16, "256 x 256 one tile per work-group (first layer narrower than 128)"),
    ("bf16", [256, 256], 130, 16, 32, "generated operand feeding the output unit, two row tiles per scenario"),
])
def test_scores_and_choices(dtype, hidden, S, P, Q, what):
    w = wl.make_scoring("grids", S, 6, hidden, P, Q, 16e3, 64e6, 1.0, 16.0, False, dtype, seed=S * 11 + P)
    part, cred = draw_grids(S, P, Q, seed=S + Q)
    desc = ab.desc_from_workload(w)
    params = ab.Params.from_workload(w, DEV)
    Cn = P * Q
    scores = torch.full((S, Cn), float("nan"), dtype=torch.float32, device=DEV)
    idx = torch.full((S,), -7, dtype=torch.int32, device=DEV)
    best = torch.full((S,), float("nan"), dtype=torch.float32, device=DEV)
    ws = ab.alloc_workspace(desc, S, Cn, device=DEV)
    ab.ab_score_candidates(desc, params, to_dev(w.dyn), to_dev(w.scal), to_dev(part), to_dev(cred),
                           scores, idx, best, ws)
    torch.cuda.synchronize()
    ref = orc.score(oracle_model(w), w.dyn, w.scal, part, cred)
    err, frac = check_scores(dtype, scores.cpu().numpy(), idx.cpu().numpy(), ref,
                             matched_scores(w, part, cred) if dtype == "bf16" else None)
    # a repeated shared grid must give what the shared-grid call gives, bit for bit
    rep_p, rep_c = np.repeat(part[:1], S, axis=0), np.repeat(cred[:1], S, axis=0)
    s_rep = torch.empty_like(scores)
    s_shared = torch.empty_like(scores)
    ab.ab_score_candidates(desc, params, to_dev(w.dyn), to_dev(w.scal), to_dev(rep_p), to_dev(rep_c), s_rep, idx, best, ws)
    ab.ab_score_candidates(desc, params, to_dev(w.dyn), to_dev(w.scal), to_dev(part[0]), to_dev(cred[0]), s_shared, idx, best, ws)
    torch.cuda.synchronize()
    same = float((s_rep - s_shared).abs().max())
    print("%s: scaled err %.3g, exact-argmax fraction %.2f, repeated-vs-shared grid max diff %.3g" % (what, err, frac, same))
    assert same <= TOL[dtype] * float(s_shared.abs().max())


@pytest.mark.parametrize("dtype,hidden,S,P,Q", [
    ("bf16", [256, 256, 256], 70, 16, 16),     # 256 x 256 streaming kernels with row-indexed candidate vectors
    ("bf16", [256, 256], 130, 16, 32),         # generated operand feeding the output unit
    ("bf16", [192, 128, 64], 50, 8, 8),        # generic tiles
    ("f32", [128], 37, 5, 7),                  # one hidden layer
    ("f32", [64, 64], 3, 8, 8),                # single launch
])
def test_integer_network_with_a_grid_per_scenario_is_reproduced_exactly(dtype, hidden, S, P, Q):
    """The exact case of the scoring tests (integer inputs, +-1 weights: nothing rounds) with every scenario
    bringing its own integer grid: scores and choices must equal the oracle's bit for bit."""
    w = wl.make_integer_scoring("int-grids", S, 6, hidden, P, Q, dtype, 500 + S, nonzeros=16)
    rng = np.random.default_rng(S + P)
    part = rng.integers(0, 4, (S, P)).astype(np.float32)
    cred = rng.integers(0, 4, (S, Q)).astype(np.float32)
    m = oracle_model(w)
    ref = orc.score(m, w.dyn, w.scal, part, cred)
    if dtype == "bf16":
        m.round_stored_bf16 = True
        assert (orc.score(m, w.dyn[:8], w.scal[:8], part[:8], cred[:8]) == ref[:8]).all()    # nothing to round
    desc = ab.desc_from_workload(w)
    params = ab.Params.from_workload(w, DEV)
    scores = torch.full((S, P * Q), float("nan"), dtype=torch.float32, device=DEV)
    idx = torch.full((S,), -7, dtype=torch.int32, device=DEV)
    best = torch.full((S,), float("nan"), dtype=torch.float32, device=DEV)
    ws = ab.alloc_workspace(desc, S, P * Q, device=DEV)
    ab.ab_score_candidates(desc, params, to_dev(w.dyn), to_dev(w.scal), to_dev(part), to_dev(cred), scores, idx, best, ws)
    torch.cuda.synchronize()
    ridx, rbest, _ = orc.select(ref)
    assert (scores.cpu().numpy() == ref.astype(np.float32)).all()
    assert (idx.cpu().numpy() == ridx).all() and (best.cpu().numpy() == rbest.astype(np.float32)).all()
