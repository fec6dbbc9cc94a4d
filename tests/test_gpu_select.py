"""ab_select_best against the oracle's sequential scan: bit-exact indices and values."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2112_13509_amd import binding as ab

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    ab.load()


def run_select(sc, C_=None, stride=None):
    t = torch.from_numpy(sc).to(DEV)
    idx = torch.full((sc.shape[0],), -9, dtype=torch.int32, device=DEV)
    best = torch.zeros(sc.shape[0], dtype=torch.float32, device=DEV)
    ab.ab_select_best(t, idx, best, C_=C_, row_stride=stride)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), best.cpu().numpy()


@pytest.mark.parametrize("S,Cn", [(1, 1), (3, 64), (17, 255), (5, 256), (9, 257), (4, 4096), (2, 5000), (1000, 33),
                                  (1001, 1024), (13, 260), (6, 1028)])
def test_random_rows_with_ties(S, Cn):
    rng = np.random.default_rng(S * 1000 + Cn)
    sc = rng.standard_normal((S, Cn)).astype(np.float32)
    sc[rng.random(sc.shape) < 0.3] = 0.5          # many exact ties
    sc[: S // 2] = np.minimum(sc[: S // 2], 0.5)  # ... that are also the maximum
    idx, best = run_select(sc)
    ridx, rbest, _ = orc.select(sc)
    assert (idx == ridx).all()
    assert (best == rbest.astype(np.float32)).all()


def test_nan_inf_and_stride():
    sc = np.array([[np.nan, 1.0, np.nan, 1.0, 0.5, 99.0],
                   [np.nan, np.nan, np.nan, np.nan, np.nan, 99.0],
                   [-np.inf, np.inf, 3.0, np.inf, 0.0, 99.0],
                   [-np.inf, -np.inf, -np.inf, -np.inf, -np.inf, 99.0]], dtype=np.float32)
    idx, best = run_select(sc, C_=5, stride=6)
    assert list(idx) == [1, -1, 1, 0]
    assert best[0] == 1.0 and np.isnan(best[1]) and best[2] == np.inf and best[3] == -np.inf


@pytest.mark.parametrize("Cn,stride", [(8, 10), (8, 12), (260, 264), (259, 264)])
def test_row_strides_of_both_alignments(Cn, stride):
    rng = np.random.default_rng(Cn * 100 + stride)
    sc = rng.standard_normal((37, stride)).astype(np.float32)
    sc[:, Cn:] = 1e9                              # beyond the row's end: must never win
    idx, best = run_select(sc, C_=Cn, stride=stride)
    ridx, rbest, _ = orc.select(np.ascontiguousarray(sc[:, :Cn]))
    assert (idx == ridx).all() and (best == rbest.astype(np.float32)).all()


def test_large_matrix_matches_oracle():
    rng = np.random.default_rng(5)
    sc = rng.standard_normal((65536, 256)).astype(np.float32)
    idx, best = run_select(sc)
    ridx, rbest, _ = orc.select(sc)
    assert (idx == ridx).all() and (best == rbest.astype(np.float32)).all()


def test_trigger_matches_oracle_bit_for_bit():
    rng = np.random.default_rng(9)
    for S, Cn, stride in [(1, 1, 1), (257, 64, 64), (1000, 300, 320), (4096, 4096, 4096)]:
        sc = (1.0 + 0.2 * rng.standard_normal((S, stride))).astype(np.float32)
        sc[rng.random(sc.shape) < 0.01] = np.nan
        if S > 3:
            sc[3, :] = np.nan
        cur = rng.integers(-1, Cn + 1, S).astype(np.int32)           # a few out-of-range indices
        obs = (1.0 + 0.2 * rng.standard_normal(S)).astype(np.float32)
        obs[rng.random(S) < 0.02] = 0.0
        t = lambda a: torch.from_numpy(a).to(DEV)
        best = torch.full((S,), -9, dtype=torch.int32, device=DEV)
        gain = torch.zeros(S, dtype=torch.float32, device=DEV)
        rec = torch.full((S,), 7, dtype=torch.uint8, device=DEV)
        ad = torch.full((S,), 7, dtype=torch.uint8, device=DEV)
        ab.ab_trigger(t(sc), t(cur), best, rec, observed=t(obs), gain=gain, adapt=ad, C_=Cn, row_stride=stride)
        torch.cuda.synchronize()
        rb, rg, rr, ra = orc.trigger(sc[:, :Cn].copy(), cur, obs)
        assert (best.cpu().numpy() == rb).all()
        g = gain.cpu().numpy()
        assert ((g == rg) | (np.isnan(g) & np.isnan(rg))).all()
        assert (rec.cpu().numpy().astype(bool) == rr).all() and (ad.cpu().numpy().astype(bool) == ra).all()
    # optional outputs may be left out
    best = torch.zeros(4, dtype=torch.int32, device=DEV)
    rec = torch.zeros(4, dtype=torch.uint8, device=DEV)
    sc = torch.tensor([[1.0, 1.06], [1.0, 1.04], [2.0, 1.0], [1.0, 1.0]], device=DEV)
    ab.ab_trigger(sc, torch.zeros(4, dtype=torch.int32, device=DEV), best, rec)
    torch.cuda.synchronize()
    assert best.tolist() == [1, 1, 0, 0] and rec.tolist() == [1, 0, 0, 0]
