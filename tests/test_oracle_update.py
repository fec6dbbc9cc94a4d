"""Pins for the oracle's online-adaptation step (Section 3.2 "Offline training online adapting";
loss per Eq. 2 read as mean squared error): finite differences, an autograd library, the closed
form of a linear model, the closed form of Adam's first step, a library Adam, training behaviour.
"""
import math

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2112_13509_amd import workloads as wl
from helpers import oracle_model


def small_problem(seed=0, L=1, hidden=(5, 4), B=7):
    u = wl.make_update("small", N=max(B, 16), batch=B, L=L, hidden=hidden, seed=seed, P=4, Q=4)
    m = oracle_model(u)
    x, y = u.x_raw[:B], u.target[:B]
    return u, m, x, y


def loss_only(m, W, b, x, y):
    st = orc.TrainState.fresh(W, b)
    return orc.update(m, st, x, y, do_adam=False, want_grads=False)["loss"]


def test_loss_is_mean_squared_error_of_the_scoring_forward():
    u, m, x, y = small_problem(1)
    st = orc.TrainState.fresh(u.W, u.b)
    out = orc.update(m, st, x, y, do_adam=False)
    # the same rows pushed through the scoring entry point: one scenario per row, 1x1 grid
    F = u.F
    for i in range(x.shape[0]):
        dyn = x[i, :F - 6].reshape(1, u.L, 3)
        sc = orc.score(m, dyn, x[i:i + 1, F - 6:F - 2], x[i, F - 2:F - 1], x[i, F - 1:F])
        assert sc[0, 0] == pytest.approx(out["yhat"][i], rel=1e-13)
    assert out["loss"] == pytest.approx(float(np.mean((out["yhat"] - y.astype(np.float64)) ** 2)), rel=1e-13)


def test_gradients_match_central_finite_differences():
    u, m, x, y = small_problem(2)
    W = [w.astype(np.float64) for w in u.W]
    b = [v.astype(np.float64) for v in u.b]
    g = orc.update(m, orc.TrainState.fresh(W, b), x, y, do_adam=False)
    checked = 0
    for k in range(len(W)):
        for arr, grad in ((W[k], g["gW"][k]), (b[k], g["gb"][k])):
            flat, gflat = arr.reshape(-1), grad.reshape(-1)
            for j in range(flat.size):
                h = 1e-6 * max(1.0, abs(flat[j]))
                old = flat[j]
                flat[j] = old + h
                lp = loss_only(m, W, b, x, y)
                flat[j] = old - h
                lm = loss_only(m, W, b, x, y)
                flat[j] = old
                fd = (lp - lm) / (2 * h)
                assert abs(fd - gflat[j]) <= 1e-6 * max(1e-3, abs(gflat[j])), (k, j, fd, gflat[j])
                checked += 1
    assert checked == sum(w.size + v.size for w, v in zip(W, b))


def _torch_forward(Wt, bt, xe):
    h = xe
    for k in range(len(Wt) - 1):
        h = torch.relu(h @ Wt[k].T + bt[k])
    return (h @ Wt[-1].T + bt[-1])[:, 0]


def _encoded_rows(m, u, x):
    F = u.F
    rows = []
    for i in range(x.shape[0]):
        X = orc.materialise_inputs(m, x[i, :F - 6].reshape(1, u.L, 3), x[i:i + 1, F - 6:F - 2],
                                   x[i, F - 2:F - 1], x[i, F - 1:F])
        rows.append(X[0, 0])
    return np.stack(rows)


def test_gradients_match_autograd():
    u, m, x, y = small_problem(3, L=2, hidden=(6, 5, 4), B=9)
    g = orc.update(m, orc.TrainState.fresh(u.W, u.b), x, y, do_adam=False)
    xe = torch.tensor(_encoded_rows(m, u, x))
    Wt = [torch.tensor(w.astype(np.float64), requires_grad=True) for w in u.W]
    bt = [torch.tensor(v.astype(np.float64), requires_grad=True) for v in u.b]
    loss = torch.mean((_torch_forward(Wt, bt, xe) - torch.tensor(y.astype(np.float64))) ** 2)
    loss.backward()
    assert g["loss"] == pytest.approx(loss.item(), rel=1e-12)
    for k in range(len(Wt)):
        np.testing.assert_allclose(g["gW"][k], Wt[k].grad.numpy(), rtol=1e-10, atol=1e-14)
        np.testing.assert_allclose(g["gb"][k], bt[k].grad.numpy(), rtol=1e-10, atol=1e-14)


def test_linear_model_gradient_closed_form():
    u, m, x, y = small_problem(4, L=2, hidden=(), B=11)
    g = orc.update(m, orc.TrainState.fresh(u.W, u.b), x, y, do_adam=False)
    X = _encoded_rows(m, u, x)
    w, b0 = u.W[0].astype(np.float64)[0], float(u.b[0][0])
    r = X @ w + b0 - y.astype(np.float64)
    np.testing.assert_allclose(g["gW"][0][0], 2.0 / 11 * X.T @ r, rtol=1e-12)
    assert g["gb"][0][0] == pytest.approx(2.0 / 11 * r.sum(), rel=1e-12)


def test_adam_first_step_closed_form():
    u, m, x, y = small_problem(5)
    st = orc.TrainState.fresh(u.W, u.b)
    before = st.copy()
    lr, eps = 1e-3, 1e-8
    out = orc.update(m, st, x, y, lr=lr, eps=eps)
    assert st.t == 1
    for k in range(len(st.W)):
        for new, old, g in ((st.W[k], before.W[k], out["gW"][k]), (st.b[k], before.b[k], out["gb"][k])):
            np.testing.assert_allclose(old - new, lr * g / (np.abs(g) + eps), rtol=1e-9, atol=1e-18)
        np.testing.assert_allclose(st.mW[k], 0.1 * out["gW"][k], rtol=1e-12)
        np.testing.assert_allclose(st.vW[k], 0.001 * out["gW"][k] ** 2, rtol=1e-9)


def test_ten_steps_match_library_adam():
    u, m, _, _ = small_problem(6, L=2, hidden=(8, 6), B=8)
    st = orc.TrainState.fresh(u.W, u.b)
    Wt = [torch.tensor(w.astype(np.float64), requires_grad=True) for w in u.W]
    bt = [torch.tensor(v.astype(np.float64), requires_grad=True) for v in u.b]
    opt = torch.optim.Adam(Wt + bt, lr=3e-3, betas=(0.8, 0.95), eps=1e-7)
    for step in range(10):
        rows = np.arange(8) + (step % 2) * 8
        x, y = u.x_raw[rows], u.target[rows]
        o = orc.update(m, st, x, y, lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-7)
        opt.zero_grad()
        loss = torch.mean((_torch_forward(Wt, bt, torch.tensor(_encoded_rows(m, u, x)))
                           - torch.tensor(y.astype(np.float64))) ** 2)
        loss.backward()
        opt.step()
        assert o["loss"] == pytest.approx(loss.item(), rel=1e-9)
    assert st.t == 10
    for k in range(len(Wt)):
        np.testing.assert_allclose(st.W[k], Wt[k].detach().numpy(), rtol=1e-8, atol=1e-12)
        np.testing.assert_allclose(st.b[k], bt[k].detach().numpy(), rtol=1e-8, atol=1e-12)


def test_forward_weights_override_only_affects_forward_backward():
    u, m, x, y = small_problem(7)
    st = orc.TrainState.fresh(u.W, u.b)
    Wq = [wl.bf16_round(w).astype(np.float64) for w in u.W]
    o = orc.update(m, st, x, y, forward_weights=Wq, do_adam=False)
    ref = orc.update(m, orc.TrainState.fresh(Wq, u.b), x, y, do_adam=False)
    assert o["loss"] == ref["loss"]
    for a, b in zip(o["gW"], ref["gW"]):
        assert (a == b).all()


def test_training_reduces_loss_towards_noise_floor():
    u = wl.make_update("train", N=2048, batch=256, L=4, hidden=(32, 32), seed=8, P=8, Q=8)
    m = oracle_model(u)
    st = orc.TrainState.fresh(u.W, u.b)
    losses = []
    for step in range(400):
        idx = u.batch_indices(step)
        losses.append(orc.update(m, st, u.x_raw[idx], u.target[idx], lr=1e-3, want_grads=False)["loss"])
    first, last = np.mean(losses[:10]), np.mean(losses[-40:])
    assert first > 5 * u.noise_var          # starts far from the target
    assert last < 0.3 * first               # and learns
    assert last > 0.5 * u.noise_var         # but cannot beat the label noise by much (it can memorise a little)


def test_minibatch_order_is_seeded_and_covers_the_pool():
    u = wl.make_update("order", N=512, batch=64, L=1, hidden=(4,), seed=9, P=2, Q=2)
    seen = np.concatenate([u.batch_indices(s) for s in range(8)])
    assert sorted(seen.tolist()) == list(range(512))
    assert (u.batch_indices(3) == u.batch_indices(3)).all()
    assert not (u.batch_indices(3) == u.batch_indices(11)).all()


def test_diagnostic_rounding_in_the_update_is_a_no_op_on_exactly_representable_values():
    """Small-integer rows, weights and targets with a batch of four: every stored activation and delta is a
    multiple of 1/2 below 128, which bfloat16 holds exactly, so the rounding-matched mode must give the plain
    oracle's loss and gradients bit for bit; with generic values it must differ, slightly."""
    rng = np.random.default_rng(17)
    L, K, B = 2, 2, 4
    lin = (0, 0.0, 1.0)
    hidden = [4, 3]
    dims = [L * K + 1 + 2] + hidden + [1]
    W = [rng.integers(-1, 2, (dims[i + 1], dims[i])).astype(np.float64) for i in range(3)]
    b = [rng.integers(0, 3, dims[i + 1]).astype(np.float64) for i in range(3)]      # (keeps units alive)
    x = rng.integers(0, 3, (B, dims[0])).astype(np.float64)
    y = rng.integers(-2, 3, B).astype(np.float64)
    m = orc.Model(L, K, [lin] * K, [lin], lin, lin, hidden, W, b)
    plain = orc.update(m, orc.TrainState.fresh(W, b), x, y, do_adam=False)
    assert max(np.abs(g).max() for g in plain["gW"]) > 0
    m.round_stored_bf16 = True
    rounded = orc.update(m, orc.TrainState.fresh(W, b), x, y, do_adam=False)
    assert rounded["loss"] == plain["loss"]
    for k in range(3):
        assert (rounded["gW"][k] == plain["gW"][k]).all() and (rounded["gb"][k] == plain["gb"][k]).all()
    # generic values
    Wg = [rng.standard_normal(w.shape) / np.sqrt(w.shape[1]) for w in W]
    xg, yg = rng.standard_normal((64, dims[0])), rng.standard_normal(64)
    m.round_stored_bf16 = False
    a = orc.update(m, orc.TrainState.fresh(Wg, b), xg, yg, do_adam=False)
    m.round_stored_bf16 = True
    c = orc.update(m, orc.TrainState.fresh(Wg, b), xg, yg, do_adam=False)
    d = max(np.abs(a["gW"][k] - c["gW"][k]).max() / np.abs(a["gW"][k]).max() for k in range(3))
    assert 0 < d < 0.1


def test_integer_network_gradients_equal_integer_arithmetic():
    """Integer rows, weights and targets, a batch of 64: with every delta scaled by B/2 the whole backward pass
    is integer arithmetic; the oracle's loss and gradients must equal the int64 evaluation exactly."""
    B = 64
    u = wl.make_integer_update("int-upd", B, 3, (24, 16), "f32", 91, n_workers=3)
    u.target = np.random.default_rng(4).integers(-5, 6, u.target.shape).astype(np.float32)
    ref = orc.update(oracle_model(u), orc.TrainState.fresh(u.W, u.b), u.x_raw, u.target, do_adam=False)
    Wi = [x.astype(np.int64) for x in u.W]
    bi = [x.astype(np.int64) for x in u.b]
    h = [u.x_raw.astype(np.int64)]
    for k in range(2):
        h.append(np.maximum(h[-1] @ Wi[k].T + bi[k], 0))
    E = h[-1] @ Wi[2].T + bi[2] - u.target.astype(np.int64)            # [B, 3]; delta_out = 2 E / B
    assert ref["loss"] == float((E * E).sum()) / B
    d = E
    for k in (2, 1, 0):
        assert (ref["gW"][k] == (d.T @ h[k]).astype(np.float64) * (2.0 / B)).all()
        assert (ref["gb"][k] == d.sum(axis=0).astype(np.float64) * (2.0 / B)).all()
        if k > 0:
            d = (d @ Wi[k]) * (h[k] > 0)
    assert np.abs(ref["gW"][0]).max() > 0
