"""Seeded random shapes through the C ABI against the oracle: depth, widths, layer count, grid, scenario count,
batch size, worker count and loss drawn from one generator, so that the hand-picked cases of the other files are
not the only corners looked at.  The measures and bounds are those of test_gpu_scoring.compare and
test_gpu_update.check_single_step."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2112_13509_amd import binding as ab
from paper_2112_13509_amd import workloads as wl
from gpu_helpers import Scorer
from test_gpu_scoring import compare
from test_gpu_update import GpuTrainer, check_single_step, TOL

pytestmark = pytest.mark.gpu
WIDTHS = [64, 128, 192, 256, 320, 512]


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    ab.load()


def scoring_cases(n=16, seed=20211213):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        dtype = "f32" if i % 2 == 0 else "bf16"
        hidden = [int(h) for h in rng.choice(WIDTHS, size=int(rng.integers(1, 5)))]
        L, P, Q = int(rng.integers(1, 41)), int(rng.integers(1, 33)), int(rng.integers(1, 33))
        S = int(rng.integers(1, 150))
        per_row = hidden[0] * (3 * L + 6) / (P * Q) + sum(a * b for a, b in zip(hidden, hidden[1:])) + hidden[-1]
        while S > 1 and S * P * Q * per_row > 6e9:       # (keeps the fp64 oracle to a few seconds)
            S //= 2
        out.append((dtype, hidden, S, L, P, Q, 7000 + i))
    return out


@pytest.mark.parametrize("dtype,hidden,S,L,P,Q,seed", scoring_cases())
def test_random_scoring_shape(dtype, hidden, S, L, P, Q, seed):
    w = wl.make_scoring("random-%d" % seed, S, L, hidden, P, Q, 16 * wl.KIB, 64 * wl.MIB, 1.0, 16.0, bool(seed & 1),
                        dtype, seed)
    print("shape: %s hidden %s, S %d, L %d, grid %d x %d" % (dtype, hidden, S, L, P, Q))
    compare(w, *Scorer(w).run(), label="random")


def update_cases(n=12, seed=20211214):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        dtype = "f32" if i % 3 else "bf16"
        hidden = tuple(int(h) for h in rng.choice(WIDTHS[:4], size=int(rng.integers(1, 5))))
        L, B = int(rng.integers(1, 30)), int(rng.integers(1, 700))
        n_workers = int(rng.choice([0, 0, 3, 16]))
        loss_kind = "l2norm" if n_workers and rng.integers(0, 2) else "mse"
        out.append((dtype, hidden, L, B, n_workers, loss_kind, 8000 + i))
    return out


@pytest.mark.parametrize("dtype,hidden,L,B,n_workers,loss_kind,seed", update_cases())
def test_random_update_shape(dtype, hidden, L, B, n_workers, loss_kind, seed):
    u = wl.make_update("random-upd-%d" % seed, N=max(2 * B, 64), batch=B, L=L, hidden=hidden, dtype=dtype, seed=seed,
                       P=8, Q=8, n_workers=n_workers, loss_kind=loss_kind)
    print("shape: %s hidden %s, L %d, B %d, workers %d, loss %s" % (dtype, hidden, L, B, n_workers, loss_kind))
    tr = GpuTrainer(u, B)
    st = orc.TrainState.fresh(u.W, u.b)
    w1 = check_single_step(u, tr, st, np.arange(B), TOL[dtype])
    w2 = check_single_step(u, tr, st, np.arange(B) + B, TOL[dtype])        # non-zero moments, other rows
    print("worst gradient error: %.3g, %.3g" % (w1, w2))
