"""Pins for the transfer-learning form of the oracle's online-adaptation step (Section 3.2 "Offline training online
adapting": the offline model is updated by transfer learning and the dataset is extended with the new samples):
frozen layers, the trainable tail against the already pinned full step, the output-layer-only case against the
closed form of linear least squares, and the replay mixing."""
import copy

import numpy as np
import torch

from oracle import oracle as orc
from test_oracle_update import small_problem


def _state(u):
    return orc.TrainState.fresh(u.W, u.b)


def test_frozen_layers_do_not_move_and_the_tail_moves_as_in_the_full_step():
    u, m, x, y = small_problem(11, hidden=(6, 5, 4), B=9)
    full = _state(u)
    out_full = orc.update(m, full, x, y, lr=1e-2)
    for k0 in range(0, 4):
        st = _state(u)
        before = copy.deepcopy(st)
        out = orc.update(m, st, x, y, lr=1e-2, first_trainable=k0)
        assert out["loss"] == out_full["loss"] and st.t == 1
        for k in range(4):
            if k < k0:
                assert np.array_equal(st.W[k], before.W[k]) and np.array_equal(st.b[k], before.b[k])
                assert not st.mW[k].any() and not st.vW[k].any() and not st.mb[k].any() and not st.vb[k].any()
                assert not out["gW"][k].any() and not out["gb"][k].any()
            else:
                # within one step the gradient of a layer does not depend on what happens below it
                assert np.array_equal(out["gW"][k], out_full["gW"][k]) and np.array_equal(out["gb"][k], out_full["gb"][k])
                assert np.array_equal(st.W[k], full.W[k]) and np.array_equal(st.b[k], full.b[k])
                assert np.array_equal(st.mW[k], full.mW[k]) and np.array_equal(st.vW[k], full.vW[k])


def test_output_layer_only_is_linear_least_squares_on_fixed_features():
    u, m, x, y = small_problem(12, hidden=(6, 5), B=8)
    st = _state(u)
    out = orc.update(m, st, x, y, do_adam=False, first_trainable=2)
    # features of the frozen body from the scoring entry point's arithmetic, re-done with a library
    F = u.F
    phi = np.empty((8, F))
    for i in range(8):
        dyn = x[i, :F - 6].reshape(1, u.L, 3)
        X = orc.materialise_inputs(m, dyn, x[i:i + 1, F - 6:F - 2], x[i, F - 2:F - 1], x[i, F - 1:F])
        phi[i] = X[0, 0]
    h = torch.from_numpy(phi)
    for k in range(2):
        h = torch.relu(h @ torch.from_numpy(u.W[k].astype(np.float64)).T + torch.from_numpy(u.b[k].astype(np.float64)))
    h = h.numpy()
    yhat = h @ u.W[2].astype(np.float64)[0] + float(u.b[2][0])
    r = 2.0 * (yhat - y.astype(np.float64)) / 8
    assert np.allclose(out["gW"][2][0], r @ h, rtol=1e-12, atol=1e-15)
    assert np.allclose(out["gb"][2][0], r.sum(), rtol=1e-12)
    assert not out["gW"][0].any() and not out["gW"][1].any()


def test_tail_training_lowers_the_loss_on_shifted_targets():
    u, m, x, y = small_problem(13, hidden=(8, 8), B=16)
    st = _state(u)
    y2 = y * 1.3 + 0.2                                      # the environment changed: speeds scale and shift
    first = orc.update(m, st, x, y2, do_adam=False, first_trainable=2)["loss"]
    for _ in range(300):
        orc.update(m, st, x, y2, lr=1e-2, first_trainable=2, want_grads=False)
    last = orc.update(m, st, x, y2, do_adam=False, first_trainable=2)["loss"]
    assert last < 0.5 * first
    assert np.array_equal(st.W[0], u.W[0].astype(np.float64)) and np.array_equal(st.W[1], u.W[1].astype(np.float64))


def test_replay_mix_picks_rows_from_both_pools():
    rng = np.random.default_rng(0)
    xn, tn = rng.standard_normal((5, 3)), rng.standard_normal(5)
    xo, to = rng.standard_normal((7, 3)), rng.standard_normal(7)
    pick = np.array([0, -1, 4, -7, 2, 2, -3, 9, -8])
    x, t = orc.replay_mix(xn, tn, xo, to, pick)
    assert np.array_equal(x[0], xn[0]) and np.array_equal(x[1], xo[0]) and np.array_equal(x[2], xn[4])
    assert np.array_equal(x[3], xo[6]) and t[3] == to[6] and np.array_equal(x[4], x[5]) and np.array_equal(x[6], xo[2])
    assert np.isnan(x[7]).all() and np.isnan(t[7]) and np.isnan(x[8]).all() and np.isnan(t[8])
    # all-new / all-old picks are plain gathers
    assert np.array_equal(orc.replay_mix(xn, tn, xo, to, np.arange(5))[0], xn)
    assert np.array_equal(orc.replay_mix(xn, tn, xo, to, -np.arange(7) - 1)[1], to)
