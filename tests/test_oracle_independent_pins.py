"""Pins that owe nothing to the oracle's own code for three things it otherwise only checks against itself
(scenarios with their own layer counts behind either encoder, a grid of its own per scenario) and for the
per-worker prediction vector V (Table 1; Eq. 1): every reference value below is computed here, in NumPy or by
a library LSTM, from the raw inputs, the model's matrices and the transform phi(x) = (g(x) - shift) * scale."""
import math

import numpy as np
import torch

from oracle import oracle as orc
from test_oracle_lstm import _model as lstm_model


def phi(x, enc):
    kind, shift, scale = enc
    return ((math.log(x) if kind == 1 else x) - shift) * scale


def relu_chain(x, Ws, bs):
    """Hidden layers with ReLU, then the linear output layer: returns the vector of all output units."""
    h = np.asarray(x, dtype=np.float64)
    for W, b in zip(Ws[:-1], bs[:-1]):
        h = np.maximum(W @ h + b, 0.0)
    return Ws[-1] @ h + bs[-1]


def mlp_model(rng, L=6, K=3, Ns=3, h0=5, h1=4, hidden=(7, 6), n_out=1):
    widths = [h1 + Ns + 2] + list(hidden) + [n_out]
    Ws = [rng.standard_normal((widths[k + 1], widths[k])) / math.sqrt(widths[k]) for k in range(len(widths) - 1)]
    bs = [0.1 * rng.standard_normal(widths[k + 1]) for k in range(len(widths) - 1)]
    te_W = [rng.standard_normal((h0, K)) / math.sqrt(K), rng.standard_normal((h1, h0)) / math.sqrt(h0)]
    te_b = [0.2 * rng.standard_normal(h0), 0.2 * rng.standard_normal(h1)]
    enc = [(1, 0.1, 0.7), (0, 0.2, 1.5), (1, -0.3, 2.0)][:K]
    scal_enc = [(0, 0.5, 2.0), (1, 0.0, 1.0), (0, 0.0, 1.0)][:Ns]
    return orc.Model(L, K, enc, scal_enc, (1, 2.0, 0.5), (0, 1.0, 0.25), list(hidden), Ws, bs,
                     te_W=te_W, te_b=te_b, te_kind="mlp")


def flat_model(rng, L=3, K=2, Ns=2, hidden=(6, 5), n_out=1):
    widths = [L * K + Ns + 2] + list(hidden) + [n_out]
    Ws = [rng.standard_normal((widths[k + 1], widths[k])) / math.sqrt(widths[k]) for k in range(len(widths) - 1)]
    bs = [0.1 * rng.standard_normal(widths[k + 1]) for k in range(len(widths) - 1)]
    return orc.Model(L, K, [(1, 0.1, 0.7), (0, 0.2, 1.5)][:K], [(0, 0.5, 2.0), (1, 0.0, 1.0)][:Ns],
                     (1, 2.0, 0.5), (0, 1.0, 0.25), list(hidden), Ws, bs)


def flat_input(m, dyn_s, scal_s, p, c):
    x = [phi(dyn_s[l, k], m.stat_enc[k]) for l in range(m.L) for k in range(m.K)]
    x += [phi(scal_s[j], m.scal_enc[j]) for j in range(m.Ns)]
    return np.array(x + [phi(p, m.part_enc), phi(c, m.cred_enc)])


def test_mean_pooled_encoder_with_own_layer_counts_divides_by_the_scenarios_own_count():
    rng = np.random.default_rng(71)
    m = mlp_model(rng)
    S = 5
    dyn, scal = rng.uniform(0.5, 3.0, (S, m.L, m.K)), rng.uniform(0.5, 2.0, (S, m.Ns))
    part, cred = np.array([1e4, 1e6]), np.array([1.0, 4.0, 9.0])
    lens = np.array([6, 1, 4, 2, 5], dtype=np.int32)
    got = orc.score(m, dyn, scal, part, cred, layers_of=lens)
    for s in range(S):
        n = int(lens[s])
        pooled = np.zeros(m.te_W[1].shape[0])
        for l in range(n):                                            # the scenario's own layers only
            x = np.array([phi(dyn[s, l, k], m.stat_enc[k]) for k in range(m.K)])
            h = np.maximum(m.te_W[0] @ x + m.te_b[0], 0.0)
            pooled += np.maximum(m.te_W[1] @ h + m.te_b[1], 0.0)
        pooled /= n                                                   # explicit division by its own count
        sc = [phi(scal[s, j], m.scal_enc[j]) for j in range(m.Ns)]
        for ip, p in enumerate(part):
            for iq, c in enumerate(cred):
                x = np.concatenate([pooled, sc, [phi(p, m.part_enc), phi(c, m.cred_enc)]])
                want = relu_chain(x, m.W, m.b)[0]
                assert abs(got[s, ip * len(cred) + iq] - want) <= 1e-12 * max(1.0, abs(want)), (s, ip, iq)


def test_lstm_encoder_with_own_layer_counts_is_a_library_lstm_on_the_truncated_sequence():
    rng = np.random.default_rng(72)
    m = lstm_model(rng, L=9)
    E, H, S = 5, 4, 6
    dyn = rng.uniform(0.5, 3.0, (S, m.L, m.K))
    lens = np.array([9, 1, 5, 3, 8, 2], dtype=np.int32)
    got = orc.lstm_encode(m, dyn, layers_of=lens)
    lib = torch.nn.LSTM(E, H, num_layers=2, batch_first=True).double()
    with torch.no_grad():
        for layer, (W, b, nx) in enumerate(((m.te_W[1], m.te_b[1], E), (m.te_W[2], m.te_b[2], H))):
            getattr(lib, "weight_ih_l%d" % layer).copy_(torch.from_numpy(W[:, :nx].copy()))
            getattr(lib, "weight_hh_l%d" % layer).copy_(torch.from_numpy(W[:, nx:].copy()))
            getattr(lib, "bias_ih_l%d" % layer).copy_(torch.from_numpy(b))
            getattr(lib, "bias_hh_l%d" % layer).zero_()
        for s in range(S):
            n = int(lens[s])
            x = np.array([[phi(dyn[s, l, k], m.stat_enc[k]) for k in range(m.K)] for l in range(n)])
            emb = x @ m.te_W[0].T + m.te_b[0]
            _, (hn, _) = lib(torch.from_numpy(emb[None]))
            assert np.abs(got[s] - hn[1, 0].numpy()).max() < 1e-13, s


def test_per_scenario_grids_against_a_numpy_chain_on_inputs_built_here():
    rng = np.random.default_rng(73)
    m = flat_model(rng)
    S, P, Q = 4, 3, 2
    dyn, scal = rng.uniform(0.5, 3.0, (S, m.L, m.K)), rng.uniform(0.5, 2.0, (S, m.Ns))
    part = np.exp(rng.uniform(np.log(16e3), np.log(64e6), (S, P)))
    cred = rng.uniform(1.0, 16.0, (S, Q))
    got = orc.score(m, dyn, scal, part, cred)
    assert got.shape == (S, P * Q)
    for s in range(S):
        for p in range(P):
            for q in range(Q):
                want = relu_chain(flat_input(m, dyn[s], scal[s], part[s, p], cred[s, q]), m.W, m.b)[0]
                assert abs(got[s, p * Q + q] - want) <= 1e-12 * max(1.0, abs(want)), (s, p, q)


def test_predicted_speed_vector_of_one_candidate_per_scenario():
    rng = np.random.default_rng(74)
    m = flat_model(rng, n_out=5)
    S, P, Q = 6, 3, 4
    dyn, scal = rng.uniform(0.5, 3.0, (S, m.L, m.K)), rng.uniform(0.5, 2.0, (S, m.Ns))
    part, cred = np.array([1e4, 1e6, 3e7]), np.array([1.0, 2.0, 4.0, 9.0])
    cand = np.array([0, 11, 5, -1, 12, 7], dtype=np.int32)           # -1 and 12 are no candidates
    V = orc.predict_v(m, dyn, scal, part, cred, cand)
    assert V.shape == (S, 5)
    scores = orc.score(m, dyn, scal, part, cred)
    for s in range(S):
        if cand[s] < 0 or cand[s] >= P * Q:
            assert np.isnan(V[s]).all()
            continue
        p, q = divmod(int(cand[s]), Q)
        want = relu_chain(flat_input(m, dyn[s], scal[s], part[p], cred[q]), m.W, m.b)
        assert np.abs(V[s] - want).max() <= 1e-12
        assert abs(V[s].mean() - scores[s, cand[s]]) <= 1e-12          # candidates are ranked by the mean of V
    # a grid of its own per scenario
    part_s = np.exp(rng.uniform(np.log(16e3), np.log(64e6), (S, P)))
    cred_s = rng.uniform(1.0, 16.0, (S, Q))
    Vs = orc.predict_v(m, dyn, scal, part_s, cred_s, np.full(S, 6, np.int32))
    for s in range(S):
        want = relu_chain(flat_input(m, dyn[s], scal[s], part_s[s, 1], cred_s[s, 2]), m.W, m.b)
        assert np.abs(Vs[s] - want).max() <= 1e-12
