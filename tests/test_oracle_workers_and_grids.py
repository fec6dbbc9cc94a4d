"""Pins for the oracle's per-worker output (Table 1: V has one entry per worker), the unsquared L2 loss of
Eq. 2, and per-scenario candidate grids: a library matmul chain, linearity of the mean, central finite
differences, an autograd library, the closed form of a linear model under the absolute-error loss, and
agreement with scenario-by-scenario calls of the shared-grid scorer.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2112_13509_amd import workloads as wl
from helpers import oracle_model
from test_oracle_update import _encoded_rows


def worker_problem(seed, n_workers, loss_kind, L=2, hidden=(6, 5), B=9):
    u = wl.make_update("workers", N=max(B, 16), batch=B, L=L, hidden=hidden, seed=seed, P=4, Q=4,
                       n_workers=n_workers, loss_kind=loss_kind)
    return u, oracle_model(u), u.x_raw[:B], u.target[:B]


def test_score_of_a_vector_output_is_the_mean_of_a_library_chain():
    u, m, x, _ = worker_problem(11, 5, "l2norm")
    dyn = x[:, :u.F - 6].reshape(-1, u.L, 3)
    scal = x[:, u.F - 6:u.F - 2]
    part, cred = np.array([1e5, 1e6, 4e6]), np.array([1.0, 2.0, 8.0, 16.0])
    got = orc.score(m, dyn, scal, part, cred)
    X = orc.materialise_inputs(m, dyn, scal, part, cred).reshape(-1, u.F)
    h = X
    for k in range(len(u.hidden)):
        h = np.maximum(h @ u.W[k].astype(np.float64).T + u.b[k], 0.0)
    V = h @ u.W[-1].astype(np.float64).T + u.b[-1]
    assert V.shape[1] == 5
    np.testing.assert_allclose(got.reshape(-1), V.mean(axis=1), rtol=1e-12, atol=1e-14)
    # linearity: the same scores from a single output unit that holds the mean of the five
    folded = oracle_model(u, W=list(u.W[:-1]) + [u.W[-1].astype(np.float64).mean(axis=0, keepdims=True)],
                          b=list(u.b[:-1]) + [np.array([u.b[-1].astype(np.float64).mean()])])
    np.testing.assert_allclose(orc.score(folded, dyn, scal, part, cred), got, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("n_workers,loss_kind", [(3, "l2norm"), (1, "l2norm"), (4, "mse")])
def test_loss_value_and_central_finite_differences(n_workers, loss_kind):
    u, m, x, y = worker_problem(20 + n_workers, n_workers, loss_kind, L=1, hidden=(5, 4), B=7)
    W = [w.astype(np.float64) for w in u.W]
    b = [v.astype(np.float64) for v in u.b]
    y2 = y.reshape(7, -1).astype(np.float64)

    def loss_only():
        return orc.update(m, orc.TrainState.fresh(W, b), x, y2, do_adam=False, want_grads=False)["loss"]

    g = orc.update(m, orc.TrainState.fresh(W, b), x, y2, do_adam=False)
    err = g["yhat"].reshape(7, -1) - y2
    want = np.mean(np.sqrt((err ** 2).sum(axis=1))) if loss_kind == "l2norm" else np.mean((err ** 2).sum(axis=1))
    assert g["loss"] == pytest.approx(float(want), rel=1e-13)
    for k in range(len(W)):
        for arr, grad in ((W[k], g["gW"][k]), (b[k], g["gb"][k])):
            flat, gflat = arr.reshape(-1), grad.reshape(-1)
            for j in range(flat.size):
                h = 1e-6 * max(1.0, abs(flat[j]))
                old = flat[j]
                flat[j] = old + h
                lp = loss_only()
                flat[j] = old - h
                lm = loss_only()
                flat[j] = old
                fd = (lp - lm) / (2 * h)
                assert abs(fd - gflat[j]) <= 2e-6 * max(1e-3, abs(gflat[j])), (k, j, fd, gflat[j])


def test_l2norm_gradients_match_autograd():
    u, m, x, y = worker_problem(31, 4, "l2norm", L=2, hidden=(6, 5, 4), B=9)
    g = orc.update(m, orc.TrainState.fresh(u.W, u.b), x, y, do_adam=False)
    xe = torch.tensor(_encoded_rows(m, u, x))
    Wt = [torch.tensor(w.astype(np.float64), requires_grad=True) for w in u.W]
    bt = [torch.tensor(v.astype(np.float64), requires_grad=True) for v in u.b]
    h = xe
    for k in range(len(Wt) - 1):
        h = torch.relu(h @ Wt[k].T + bt[k])
    out = h @ Wt[-1].T + bt[-1]
    loss = torch.linalg.vector_norm(out - torch.tensor(y.astype(np.float64)), dim=1).mean()
    loss.backward()
    assert g["loss"] == pytest.approx(loss.item(), rel=1e-12)
    for k in range(len(Wt)):
        np.testing.assert_allclose(g["gW"][k], Wt[k].grad.numpy(), rtol=1e-10, atol=1e-14)
        np.testing.assert_allclose(g["gb"][k], bt[k].grad.numpy(), rtol=1e-10, atol=1e-14)


def test_single_output_l2norm_is_the_absolute_error_closed_form():
    u, m, x, y = worker_problem(41, 1, "l2norm", L=2, hidden=(), B=11)
    g = orc.update(m, orc.TrainState.fresh(u.W, u.b), x, y, do_adam=False)
    X = _encoded_rows(m, u, x)
    r = X @ u.W[0].astype(np.float64)[0] + float(u.b[0][0]) - y[:, 0].astype(np.float64)
    assert g["loss"] == pytest.approx(float(np.abs(r).mean()), rel=1e-13)
    np.testing.assert_allclose(g["gW"][0][0], X.T @ np.sign(r) / 11, rtol=1e-12)
    assert g["gb"][0][0] == pytest.approx(np.sign(r).sum() / 11, rel=1e-12)


def test_zero_error_rows_contribute_no_gradient_under_the_norm_loss():
    u, m, x, y = worker_problem(51, 3, "l2norm", L=1, hidden=(4,), B=6)
    st = orc.TrainState.fresh(u.W, u.b)
    yhat = orc.update(m, st, x, y, do_adam=False)["yhat"]
    y2 = y.astype(np.float64).copy()
    y2[:3] = yhat[:3]                                         # three rows predicted exactly
    g_all = orc.update(m, st, x, y2, do_adam=False)
    g_rest = orc.update(m, st, x[3:], y2[3:], do_adam=False)  # the other three alone, mean over 3 instead of 6
    for k in range(len(st.W)):
        np.testing.assert_allclose(g_all["gW"][k], g_rest["gW"][k] * 0.5, rtol=1e-10, atol=1e-15)


def test_per_scenario_grids_equal_scenario_by_scenario_calls():
    w = wl.make_config(1, S=5)
    m = oracle_model(w)
    rng = np.random.default_rng(3)
    part = np.exp(rng.uniform(np.log(16e3), np.log(64e6), size=(5, 3)))
    cred = rng.uniform(1.0, 16.0, size=(5, 4))
    got = orc.score(m, w.dyn, w.scal, part, cred)
    assert got.shape == (5, 12)
    for s in range(5):
        one = orc.score(m, w.dyn[s:s + 1], w.scal[s:s + 1], part[s], cred[s])
        assert (one[0] == got[s]).all()
    # a grid repeated for every scenario is the shared grid
    shared = orc.score(m, w.dyn, w.scal, part[0], cred[0])
    rep = orc.score(m, w.dyn, w.scal, np.repeat(part[:1], 5, axis=0), np.repeat(cred[:1], 5, axis=0))
    assert (shared == rep).all()
