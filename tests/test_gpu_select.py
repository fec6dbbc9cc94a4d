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


@pytest.mark.parametrize("S,Cn", [(1, 1), (3, 64), (17, 255), (5, 256), (9, 257), (4, 4096), (2, 5000), (1000, 33)])
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


def test_large_matrix_matches_oracle():
    rng = np.random.default_rng(5)
    sc = rng.standard_normal((65536, 256)).astype(np.float32)
    idx, best = run_select(sc)
    ridx, rbest, _ = orc.select(sc)
    assert (idx == ridx).all() and (best == rbest.astype(np.float32)).all()
