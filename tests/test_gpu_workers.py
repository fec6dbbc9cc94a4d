"""Per-worker prediction V (one output unit per worker, Table 1) and the unsquared L2 loss of Eq. 2 on the
GPU against the oracle: scoring ranks candidates by the mean of the per-worker predictions, the update
back-propagates the chosen loss through the n-wide output layer."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2112_13509_amd import binding as ab
from paper_2112_13509_amd import workloads as wl
from helpers import oracle_model
from gpu_helpers import Scorer, check_scores, matched_scores
from test_gpu_update import GpuTrainer, check_single_step, TOL

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    ab.load()


def with_worker_outputs(w, n_workers, seed):
    """The scoring workload with its output layer redrawn as n_workers units (weights N(0, 1/fan_in))."""
    rng = np.random.default_rng(seed)
    H = w.hidden[-1]
    Wo = (rng.standard_normal((n_workers, H)) / np.sqrt(H)).astype(np.float32)
    if w.dtype == "bf16":
        Wo = wl.bf16_round(Wo)
    w.W = list(w.W[:-1]) + [Wo]
    w.b = list(w.b[:-1]) + [(0.1 * rng.standard_normal(n_workers)).astype(np.float32)]
    return w


@pytest.mark.parametrize("dtype,hidden,S,P,Q,n_workers", [
    ("f32", [64, 64], 9, 8, 8, 4),            # generic tiles
    ("bf16", [128], 33, 5, 7, 3),             # single hidden layer
    ("bf16", [256, 256, 256], 70, 16, 16, 8),  # 256 x 256 streaming kernels (70 tiles per launch)
    ("f32", [64, 64], 1, 8, 8, 16),           # a size the single-launch path would take with one output
])
def test_scores_are_the_mean_of_the_per_worker_predictions(dtype, hidden, S, P, Q, n_workers):
    w = wl.make_scoring("workers", S, 6, hidden, P, Q, 16e3, 64e6, 1.0, 16.0, False, dtype, seed=S * 7 + n_workers)
    w = with_worker_outputs(w, n_workers, seed=n_workers)
    sc = Scorer(w)
    assert sc.desc.n_outputs == n_workers
    scores, idx, best = sc.run()
    ref = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
    err, frac = check_scores(dtype, scores, idx, ref, matched_scores(w) if dtype == "bf16" else None)
    print("n_workers=%d %s: scaled err %.3g, exact-argmax fraction %.2f" % (n_workers, dtype, err, frac))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_workers,loss_kind", [(1, "l2norm"), (3, "l2norm"), (8, "l2norm"), (16, "l2norm"), (4, "mse")])
def test_single_update_step(dtype, n_workers, loss_kind):
    B = 300
    u = wl.make_update("upd-workers", N=512, batch=B, L=5, hidden=(128, 64), dtype=dtype, seed=n_workers * 10 + 1,
                       P=8, Q=8, n_workers=n_workers, loss_kind=loss_kind)
    tr = GpuTrainer(u, B)
    assert tr.desc.n_outputs == n_workers and tr.desc.loss_kind == (1 if loss_kind == "l2norm" else 0)
    st = orc.TrainState.fresh(u.W, u.b)
    w1 = check_single_step(u, tr, st, np.arange(B), TOL[dtype])
    w2 = check_single_step(u, tr, st, np.arange(B)[::-1].copy() + 100, TOL[dtype])
    print("%s n_workers=%d %s: worst gradient error %.3g, %.3g" % (dtype, n_workers, loss_kind, w1, w2))


def test_norm_loss_at_the_real_shape_bf16():
    """Configuration 4's network and batch with eight workers and the norm loss."""
    u = wl.make_update("cfg4-workers", N=4096, batch=4096, n_workers=8, loss_kind="l2norm")
    tr = GpuTrainer(u, 4096)
    st = orc.TrainState.fresh(u.W, u.b)
    w = check_single_step(u, tr, st, np.arange(4096), TOL["bf16"])
    print("cfg4 shape, 8 workers, norm loss: worst gradient error %.3g" % w)


def test_a_row_predicted_exactly_gives_no_gradient_and_no_nan():
    u = wl.make_update("upd-exact", N=64, batch=64, L=2, hidden=(64,), dtype="f32", seed=5, P=4, Q=4,
                       n_workers=2, loss_kind="l2norm")
    tr = GpuTrainer(u, 64)
    # zero output layer and zero targets: every error vector is exactly zero
    u.W[-1][:] = 0.0
    u.b[-1][:] = 0.0
    u.target[:] = 0.0
    tr = GpuTrainer(u, 64)
    st = orc.TrainState.fresh(u.W, u.b)
    tr.load_state(st)
    tr.step(np.arange(64))
    assert tr.loss_value() == 0.0
    for k in range(len(st.W)):
        assert torch.equal(tr.params.mW[k], torch.zeros_like(tr.params.mW[k]))
        assert torch.isfinite(tr.params.W_master[k]).all()


@pytest.mark.parametrize("dtype,S,L,hidden", [("f32", 40, 12, [128, 64]), ("bf16", 300, 48, [256, 256, 256])])
def test_table1_record_with_per_worker_inputs_and_outputs(dtype, S, L, hidden):
    """Eight workers: T is L x 8, B_d and B_u have eight entries each (22 scalars), V has eight entries."""
    w = wl.make_per_worker("table1", S, L, 8, hidden, 16, 16, dtype, seed=S + L)
    sc = Scorer(w)
    assert sc.desc.n_stats == 8 and sc.desc.n_scalars == 22 and sc.desc.n_outputs == 8
    scores, idx, best = sc.run()
    ref = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
    err, frac = check_scores(dtype, scores, idx, ref, matched_scores(w) if dtype == "bf16" else None)
    print("Table 1 record %s: err %.3g, exact-argmax fraction %.2f" % (dtype, err, frac))


@pytest.mark.parametrize("dtype,hidden,S,P,Q,n_workers", [
    ("bf16", [256, 256, 256], 70, 16, 16, 8),
    ("bf16", [128, 64], 40, 5, 7, 16),
    ("f32", [64, 64], 9, 8, 8, 4),
])
def test_integer_network_with_per_worker_outputs_is_reproduced_exactly(dtype, hidden, S, P, Q, n_workers):
    """The exact case (integer inputs, +-1 weights) with a power-of-two number of output units: the mean of the
    per-worker predictions is a multiple of 1 / n_workers, nothing rounds, and scores and choices must equal the
    oracle's bit for bit although the library folds the output layer into one unit and the oracle does not."""
    w = wl.make_integer_scoring("int-workers", S, 6, hidden, P, Q, dtype, 700 + S, nonzeros=16)
    rng = np.random.default_rng(n_workers)
    w.W = list(w.W[:-1]) + [rng.integers(-1, 2, (n_workers, hidden[-1])).astype(np.float32)]
    w.b = list(w.b[:-1]) + [rng.integers(-2, 3, n_workers).astype(np.float32)]
    m = oracle_model(w)
    ref = orc.score(m, w.dyn, w.scal, w.part, w.cred)
    if dtype == "bf16":
        m.round_stored_bf16 = True
        assert (orc.score(m, w.dyn, w.scal, w.part, w.cred) == ref).all()
    assert (ref * n_workers == np.round(ref * n_workers)).all() and len(np.unique(ref)) > 8
    sc = Scorer(w)
    scores, idx, best = sc.run()
    ridx, rbest, _ = orc.select(ref)
    assert (scores == ref.astype(np.float32)).all()
    assert (idx == ridx).all() and (best == rbest.astype(np.float32)).all()
    # the chosen candidate's prediction vector, unfolded: integers, so equal to the oracle's bit for bit
    _, idx_v, best_v, V = sc.run(want_scores=False, want_v=True)
    assert (idx_v == ridx).all() and (best_v == best).all()
    assert (V == orc.predict_v(oracle_model(w), w.dyn, w.scal, w.part, w.cred, ridx).astype(np.float32)).all()
    assert len(np.unique(V)) > 4 and (V.mean(axis=1, dtype=np.float64) == rbest).all()


@pytest.mark.parametrize("dtype,hidden,S,P,Q,n_workers,per_scenario", [
    ("f32", [64, 64], 3, 8, 8, 4, False),              # a size the single-launch path would take without the vector
    ("f32", [128], 33, 5, 7, 3, False),                # one hidden layer: the vector comes straight from the scenario term
    ("bf16", [64], 20, 4, 4, 16, True),
    ("bf16", [256, 256, 256], 70, 16, 16, 8, False),   # 256 x 256 streaming kernels in the scoring pass
    ("bf16", [512, 512], 40, 32, 32, 16, True),        # a grid of its own per scenario
    ("bf16", [128, 256, 128, 64], 9, 6, 6, 1, False),  # one output: the vector is the best score itself
    ("bf16", [1024] * 4, 4100, 16, 16, 8, False),      # more scenarios than one chunk of the second pass holds
])
def test_prediction_vector_of_the_chosen_candidate(dtype, hidden, S, P, Q, n_workers, per_scenario):
    """ab_score_candidates_v: V (one entry per worker, Table 1; Eq. 1) of the candidate the pass chose, against the
    oracle's unfolded forward pass for that same candidate."""
    w = wl.make_scoring("v-best", S, 6, hidden, P, Q, 16e3, 64e6, 1.0, 16.0, False, dtype, seed=S * 3 + n_workers)
    w = with_worker_outputs(w, n_workers, seed=n_workers + 1)
    part, cred = w.part, w.cred
    if per_scenario:
        rng = np.random.default_rng(S)
        part = np.exp(rng.uniform(np.log(16e3), np.log(64e6), (S, P))).astype(np.float32)
        cred = rng.uniform(1.0, 16.0, (S, Q)).astype(np.float32)
    sc = Scorer(w)
    scores, idx, best, V = sc.run(want_v=True, part=part, cred=cred)
    assert V.shape == (S, n_workers) and np.isfinite(V).all()
    m = oracle_model(w)
    ref = orc.predict_v(m, w.dyn, w.scal, part, cred, idx)            # the candidate the GPU chose
    scale = np.abs(ref).max()
    err = np.abs(V - ref).max() / scale
    mean_gap = np.abs(V.mean(axis=1, dtype=np.float64) - best).max() / max(np.abs(best).max(), 1e-30)
    msg = "V of the chosen candidate %s %s: max err %.3g of max |V|, |mean V - best score| %.3g" % (dtype, hidden, err, mean_gap)
    if dtype == "bf16":
        m.round_stored_bf16 = True
        errq = np.abs(V - orc.predict_v(m, w.dyn, w.scal, part, cred, idx)).max() / scale
        msg += ", vs rounding-matched oracle %.3g" % errq
        assert errq <= (2e-3 if len(hidden) <= 2 else 1e-2), msg
    print(msg)
    assert err <= TOL[dtype], msg
    assert mean_gap <= (1e-5 if dtype == "f32" else 1e-2), msg
    # same choice and scores as the plain entry point
    s2, i2, b2 = sc.run(part=part, cred=cred)
    if not (dtype == "f32" and S * P * Q <= 16384 and max(hidden) <= 128):     # (the single-launch path sums differently)
        assert np.array_equal(s2, scores) and np.array_equal(i2, idx) and np.array_equal(b2, best)


def test_prediction_vector_is_nan_where_nothing_could_be_chosen():
    w = wl.make_scoring("v-nan", 6, 8, [64, 64], 4, 4, 16e3, 64e6, 1.0, 16.0, False, "f32", seed=5)
    w = with_worker_outputs(w, 3, seed=2)
    w.dyn[2, 1, 0] = np.nan
    _, idx, best, V = Scorer(w).run(want_v=True)
    assert idx[2] == -1 and np.isnan(V[2]).all()
    ok = [0, 1, 3, 4, 5]
    ref = orc.predict_v(oracle_model(w), w.dyn, w.scal, w.part, w.cred, idx)
    assert np.isnan(ref[2]).all() and np.abs(V[ok] - ref[ok]).max() <= 1e-4 * np.abs(ref[ok]).max()


@pytest.mark.parametrize("dtype,S,L,hidden", [("f32", 40, 12, [128, 64]), ("bf16", 300, 48, [256, 256, 256])])
def test_table1_record_of_a_sixteen_worker_job(dtype, S, L, hidden):
    """Sixteen workers: T is L x 16 (sixteen statistics per layer), B_d and B_u have sixteen entries each (38
    scalars), V has sixteen entries; scores, choice and the chosen candidate's V against the oracle."""
    w = wl.make_per_worker("table1-16", S, L, 16, hidden, 16, 16, dtype, seed=S + L + 16)
    sc = Scorer(w)
    assert sc.desc.n_stats == 16 and sc.desc.n_scalars == 38 and sc.desc.n_outputs == 16
    scores, idx, best, V = sc.run(want_v=True)
    ref = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
    err, frac = check_scores(dtype, scores, idx, ref, matched_scores(w) if dtype == "bf16" else None)
    refv = orc.predict_v(oracle_model(w), w.dyn, w.scal, w.part, w.cred, idx)
    errv = np.abs(V - refv).max() / np.abs(refv).max()
    print("Table 1 record, 16 workers, %s: score err %.3g, exact-argmax fraction %.2f, V err %.3g" % (dtype, err, frac, errv))
    assert errv <= TOL[dtype]
