"""The scorer without hidden layers (V = W x + b) on the GPU: the closed form that pins the oracle's selection
(a one-layer linear network picks the same grid corner for every scenario, given by the signs of the two
configuration weights; with both zero every score ties and index 0 wins), scores, choice and per-worker vector
against the oracle, and the update step against the oracle's (whose gradient is the closed form
(2/B) X^T (X w + b - y), pinned in tests/test_oracle_update.py)."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2112_13509_amd import binding as ab
from paper_2112_13509_amd import workloads as wl
from helpers import oracle_model, scaled_error, tensor_scaled_error, check_selection, tensor_error
from gpu_helpers import Scorer

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    ab.load()


def linear_workload(S, L, P, Q, dtype, seed, n_out=1):
    w = wl.make_scoring("linear", S, L, [], P, Q, 16 * wl.KIB, 64 * wl.MIB, 1.0, 64.0, False, dtype, seed)
    if n_out > 1:
        rng = np.random.default_rng(seed + 1)
        W = (rng.standard_normal((n_out, w.F)) / np.sqrt(w.F)).astype(np.float32)
        w.W = [wl.bf16_round(W) if dtype == "bf16" else W]
        w.b = [(0.1 * rng.standard_normal(n_out)).astype(np.float32)]
    return w


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("sp,sc", [(1, 1), (1, -1), (-1, 1), (-1, -1), (0, 0)])
def test_one_layer_network_picks_the_grid_corner_its_weight_signs_name(dtype, sp, sc):
    P, Q = 6, 5
    w = linear_workload(9, 7, P, Q, dtype, 11)
    assert ab.desc_from_workload(w).n_hidden == 0
    w.W[0][0, -2] = 0.5 * sp
    w.W[0][0, -1] = 0.25 * sc
    scores, idx, best = Scorer(w).run()
    # phi is increasing in S_p and S_c, so the largest score sits at the corner the signs point to
    want = (P - 1 if sp > 0 else 0) * Q + (Q - 1 if sc > 0 else 0)
    assert (idx == want).all()
    ref = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
    assert (orc.select(ref)[0] == want).all()
    if sp == 0:
        assert (scores == scores[:, :1]).all()          # every candidate ties: the lowest index wins


@pytest.mark.parametrize("dtype,S,L,P,Q,n_out,per_scenario", [
    ("f32", 1, 16, 8, 8, 1, False), ("f32", 70, 128, 64, 64, 4, False), ("bf16", 33, 40, 16, 16, 1, True),
    ("bf16", 300, 128, 5, 7, 16, False),
])
def test_scores_choice_and_prediction_vector_against_the_oracle(dtype, S, L, P, Q, n_out, per_scenario):
    w = linear_workload(S, L, P, Q, dtype, 100 + S, n_out)
    part, cred = w.part, w.cred
    if per_scenario:
        rng = np.random.default_rng(S)
        part = np.exp(rng.uniform(np.log(16e3), np.log(64e6), (S, P))).astype(np.float32)
        cred = rng.uniform(1.0, 16.0, (S, Q)).astype(np.float32)
    scores, idx, best, V = Scorer(w).run(want_v=True, part=part, cred=cred)
    m = oracle_model(w)
    ref = orc.score(m, w.dyn, w.scal, part, cred)
    err = scaled_error(scores, ref) if dtype == "f32" else tensor_scaled_error(scores, ref)
    active = check_selection(idx, ref, TOL[dtype])
    refv = orc.predict_v(m, w.dyn, w.scal, part, cred, idx)
    errv = np.abs(V - refv).max() / np.abs(refv).max()
    msg = "linear scorer %s S=%d n_out=%d: score err %.3g, V err %.3g, exact-index check on %.0f%%" % (
        dtype, S, n_out, err, errv, 100 * active)
    if dtype == "bf16":
        m.round_stored_bf16 = True
        errq = scaled_error(scores, orc.score(m, w.dyn, w.scal, part, cred))
        msg += ", vs rounding-matched oracle %.3g" % errq
        assert errq <= 2e-3, msg                      # (a transformed input may land on the other side of a bf16 boundary)
    print(msg)
    assert err <= TOL[dtype] and errv <= TOL[dtype], msg
    assert np.array_equal(idx, np.argmax(scores, axis=1)) and np.array_equal(best, scores[np.arange(S), idx])
    assert np.abs(V.mean(axis=1, dtype=np.float64) - best).max() <= 1e-5 * max(1.0, np.abs(best).max())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_integer_linear_scorer_is_reproduced_exactly(dtype):
    w = wl.make_integer_scoring("int-linear", 50, 9, [], 7, 5, dtype, 77, nonzeros=16)
    ref = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
    scores, idx, best = Scorer(w).run()
    ridx, rbest, _ = orc.select(ref)
    assert (scores == ref.astype(np.float32)).all() and (idx == ridx).all() and (best == rbest.astype(np.float32)).all()


@pytest.mark.parametrize("dtype,n_workers,loss_kind", [("f32", 0, "mse"), ("bf16", 0, "mse"), ("f32", 4, "l2norm"),
                                                       ("bf16", 8, "mse")])
def test_update_step_of_the_linear_scorer(dtype, n_workers, loss_kind):
    from test_gpu_update import GpuTrainer, check_single_step
    B = 300
    u = wl.make_update("upd-linear", N=512, batch=B, L=20, hidden=(), dtype=dtype, seed=31 + n_workers, P=8, Q=8,
                       n_workers=n_workers, loss_kind=loss_kind)
    tr = GpuTrainer(u, B)
    assert tr.desc.n_hidden == 0
    st = orc.TrainState.fresh(u.W, u.b)
    w1 = check_single_step(u, tr, st, np.arange(B), TOL[dtype])
    w2 = check_single_step(u, tr, st, np.arange(B)[::-1].copy() + 200, TOL[dtype])      # non-zero moments
    print("linear scorer update %s n_workers=%d %s: worst gradient error %.3g, %.3g" % (dtype, n_workers, loss_kind, w1, w2))
    # closed form of the squared-error gradient on the GPU's own numbers (one output): (2/B) X^T (yhat - y)
    if n_workers == 0 and dtype == "f32":
        tr.load_state(st)
        before = st.copy()
        rows = np.arange(B)
        tr.step(rows)
        torch.cuda.synchronize()
        X = orc.materialise_inputs(oracle_model(u), u.x_raw[rows, :-6].reshape(B, u.L, 3), u.x_raw[rows, -6:-2],
                                   np.array([1.0]), np.array([1.0]))[:, 0, :]
        for i, r in enumerate(rows):                 # the row's own configuration columns
            X[i, -2] = orc.encode_value(float(u.x_raw[r, -2]), u.part_enc)
            X[i, -1] = orc.encode_value(float(u.x_raw[r, -1]), u.cred_enc)
        resid = X @ before.W[0][0] + before.b[0][0] - u.target[rows].astype(np.float64)
        g_closed = 2.0 / B * X.T @ resid
        g_gpu = (tr.params.mW[0].cpu().numpy().astype(np.float64)[0] - 0.9 * before.mW[0][0]) / 0.1
        assert tensor_error(g_gpu, g_closed) <= 1e-4
