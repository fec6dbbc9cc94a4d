"""Pins for the oracle's temporal encoder (Section 3.1 "Meta network architecture": layer-wise statistics embedded
into a fixed width, then a two-layer LSTM over the layer sequence): a library LSTM, closed forms, order of the
sequence, and the way its output enters the scorer."""
import math

import numpy as np
import torch

from oracle import oracle as orc


def _model(rng, L=7, K=3, E=5, H=4, Ns=2, hidden=(6,), zero_lstm=False):
    W_e, b_e = rng.standard_normal((E, K)), 0.1 * rng.standard_normal(E)
    W1, b1 = rng.standard_normal((4 * H, E + H)) / math.sqrt(E + H), 0.3 * rng.standard_normal(4 * H)
    W2, b2 = rng.standard_normal((4 * H, 2 * H)) / math.sqrt(2 * H), 0.3 * rng.standard_normal(4 * H)
    if zero_lstm:
        W1, W2 = np.zeros_like(W1), np.zeros_like(W2)
    widths = [H + Ns + 2] + list(hidden) + [1]
    Ws = [rng.standard_normal((widths[k + 1], widths[k])) / math.sqrt(widths[k]) for k in range(len(widths) - 1)]
    bs = [0.1 * rng.standard_normal(widths[k + 1]) for k in range(len(widths) - 1)]
    enc = [(0, 0.2, 1.5), (1, 0.1, 0.7), (0, -0.3, 2.0)][:K]
    return orc.Model(L, K, enc, [(0, 0.0, 1.0)] * Ns, (1, 2.0, 0.5), (0, 1.0, 0.25), list(hidden), Ws, bs,
                     te_W=[W_e, W1, W2], te_b=[b_e, b1, b2], te_kind="lstm")


def _phi(m, dyn):
    x = np.array(dyn, dtype=np.float64)
    for k, (kind, sh, sc) in enumerate(m.stat_enc):
        x[..., k] = ((np.log(x[..., k]) if kind == 1 else x[..., k]) - sh) * sc
    return x


def test_matches_library_lstm():
    rng = np.random.default_rng(3)
    m = _model(rng)
    E, H = 5, 4
    S = 9
    dyn = rng.uniform(0.5, 3.0, (S, m.L, m.K))
    got = orc.lstm_encode(m, dyn)
    emb = _phi(m, dyn) @ m.te_W[0].T + m.te_b[0]                                     # [S, L, E]
    lib = torch.nn.LSTM(E, H, num_layers=2, batch_first=True).double()
    with torch.no_grad():
        for layer, (W, b, nx) in enumerate(((m.te_W[1], m.te_b[1], E), (m.te_W[2], m.te_b[2], H))):
            getattr(lib, "weight_ih_l%d" % layer).copy_(torch.from_numpy(W[:, :nx].copy()))
            getattr(lib, "weight_hh_l%d" % layer).copy_(torch.from_numpy(W[:, nx:].copy()))
            getattr(lib, "bias_ih_l%d" % layer).copy_(torch.from_numpy(b))
            getattr(lib, "bias_hh_l%d" % layer).zero_()
        out, (hn, cn) = lib(torch.from_numpy(emb))
    assert np.abs(got - hn[1].numpy()).max() < 1e-13
    assert np.abs(got - out[:, -1, :].numpy()).max() < 1e-13


def test_closed_forms_without_recurrent_weights():
    rng = np.random.default_rng(4)
    H = 4
    big = 40.0
    for L, forget in ((1, -big), (6, -big), (6, big)):
        m = _model(rng, L=L, zero_lstm=True)
        beta1, beta2 = rng.standard_normal(H), rng.standard_normal(H)
        m.te_b[1] = np.concatenate([np.full(H, big), np.full(H, forget), beta1, np.full(H, big)])
        m.te_b[2] = np.concatenate([np.full(H, big), np.full(H, forget), beta2, np.full(H, big)])
        got = orc.lstm_encode(m, rng.uniform(0.5, 3.0, (3, L, m.K)))
        # input and output gates open; forget gate shut: c = tanh(beta) at every step; open: c = L tanh(beta)
        c2 = np.tanh(beta2) * (L if forget > 0 else 1)
        assert np.abs(got - np.tanh(c2)).max() < 1e-12
    # all-zero weights and biases: i = f = o = 1/2, g = 0 -> the state never leaves zero
    m = _model(rng, zero_lstm=True)
    m.te_b[1][:] = 0.0
    m.te_b[2][:] = 0.0
    assert np.abs(orc.lstm_encode(m, rng.uniform(0.5, 3.0, (2, m.L, m.K)))).max() == 0.0


def test_sequence_runs_over_the_layers_in_order():
    rng = np.random.default_rng(5)
    m = _model(rng, L=8)
    dyn = rng.uniform(0.5, 3.0, (4, m.L, m.K))
    a = orc.lstm_encode(m, dyn)
    assert np.abs(a - orc.lstm_encode(m, dyn[:, ::-1, :].copy())).max() > 1e-3      # direction matters
    # with the forget gates shut the state holds the last layer only: earlier layers may change freely
    H = 4
    m.te_b[1][H:2 * H] = -60.0
    m.te_b[2][H:2 * H] = -60.0
    m.te_W[1][:, 5:] = 0.0                                                           # no recurrent path either
    m.te_W[2][:, H:] = 0.0
    d2 = dyn.copy()
    d2[:, :-1, :] = rng.uniform(0.5, 3.0, d2[:, :-1, :].shape)
    assert np.abs(orc.lstm_encode(m, dyn) - orc.lstm_encode(m, d2)).max() < 1e-12
    d2[:, -1, :] *= 1.5
    assert np.abs(orc.lstm_encode(m, dyn) - orc.lstm_encode(m, d2)).max() > 1e-3


def test_encoder_output_is_the_statistics_block_of_the_scorer():
    rng = np.random.default_rng(6)
    m = _model(rng)
    S = 5
    dyn, scal = rng.uniform(0.5, 3.0, (S, m.L, m.K)), rng.standard_normal((S, 2))
    part, cred = np.array([1e4, 1e6, 1e7]), np.array([1.0, 4.0])
    X = orc.materialise_inputs(m, dyn, scal, part, cred)
    enc = orc.lstm_encode(m, dyn)
    assert X.shape == (S, 6, 4 + 2 + 2)
    assert np.abs(X[:, :, :4] - enc[:, None, :]).max() == 0.0
    assert np.abs(X[:, :, 4:6] - scal[:, None, :]).max() < 1e-15
    h = np.maximum(X @ m.W[0].T + m.b[0], 0.0)
    want = (h @ m.W[1].T + m.b[1])[..., 0]
    assert np.abs(orc.score(m, dyn, scal, part, cred) - want).max() < 1e-12
