"""Pins for the oracle's scoring / selection against things other than itself.

Paper passages: Table 1 (input record), Section 3.1 "Meta network architecture" (concatenate the
feature groups, dense layers, predicted V), Eq. 1, and the choice of the pair with the largest
predicted V (Section 3 intro).  The paper prints no numeric example of the meta-network, so the
pins are mathematical: brute force, a library matmul chain, closed forms and invariants.
"""
import math

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2112_13509_amd import workloads as wl
from helpers import oracle_model


# ---- an independent scalar evaluator: one candidate at a time, explicit vectors and sums -------
def _phi(x, enc):
    kind, shift, scale = enc
    g = math.log(x) if kind == 1 else x
    return (g - shift) * scale


def brute_force_score(w, s, p, q):
    x = []
    if w.te_W is None:
        for l in range(w.L):
            for k in range(w.K):
                x.append(_phi(float(w.dyn[s, l, k]), w.stat_enc[k]))
    else:
        h1n = w.te_W[1].shape[0]
        pool = [0.0] * h1n
        for l in range(w.L):
            t = [_phi(float(w.dyn[s, l, k]), w.stat_enc[k]) for k in range(w.K)]
            h0 = [max(0.0, float(w.te_b[0][o]) + sum(float(w.te_W[0][o, i]) * t[i] for i in range(w.K)))
                  for o in range(w.te_W[0].shape[0])]
            h1 = [max(0.0, float(w.te_b[1][o]) + sum(float(w.te_W[1][o, i]) * h0[i] for i in range(len(h0))))
                  for o in range(h1n)]
            pool = [a + b for a, b in zip(pool, h1)]
        x = [a / w.L for a in pool]
    for j in range(w.Ns):
        x.append(_phi(float(w.scal[s, j]), w.scal_enc[j]))
    x.append(_phi(float(w.part[p]), w.part_enc))
    x.append(_phi(float(w.cred[q]), w.cred_enc))
    h = x
    for k in range(len(w.hidden)):
        h = [max(0.0, float(w.b[k][o]) + sum(float(w.W[k][o, i]) * h[i] for i in range(len(h))))
             for o in range(w.hidden[k])]
    return float(w.b[-1][0]) + sum(float(w.W[-1][0, i]) * h[i] for i in range(len(h)))


def test_brute_force_tiny_grids():
    for seed, (L, hidden, P, Q, S) in enumerate([(2, [4, 3], 3, 2, 3), (1, [2], 2, 3, 2),
                                                 (1, [], 2, 2, 2), (3, [5, 4, 3], 1, 4, 2)]):
        w = wl.make_scoring("tiny", S, L, hidden, P, Q, 64 * wl.KIB, 64 * wl.MIB, 1.0, 8.0,
                            True, "f32", 100 + seed)
        got = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
        for s in range(S):
            for p in range(P):
                for q in range(Q):
                    ref = brute_force_score(w, s, p, q)
                    assert abs(got[s, p * Q + q] - ref) <= 1e-12 * max(1.0, abs(ref))


def test_brute_force_config1():
    w = wl.make_config(1)
    got = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
    assert got.shape == (1, 64)
    for p in range(8):
        for q in range(8):
            ref = brute_force_score(w, 0, p, q)
            assert abs(got[0, p * 8 + q] - ref) <= 1e-12 * max(1.0, abs(ref))
    # picking the best by exhaustive comparison
    best = max(range(64), key=lambda c: (got[0, c], -c))
    idx, bs, second = orc.select(got)
    assert idx[0] == best and bs[0] == got[0, best]
    assert second[0] == np.sort(got[0])[-2]


def test_brute_force_tensor_encoder():
    w = wl.make_tensor_encoder("tiny-te", 2, [4], [3, 5], 2, 2, "f32", 7, n_blocks=2, per_block=2, extra=1)
    got = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
    for s in range(2):
        for c in range(4):
            ref = brute_force_score(w, s, c // 2, c % 2)
            assert abs(got[s, c] - ref) <= 1e-12 * max(1.0, abs(ref))


# ---- library matmul chain on the explicitly materialised [S*C, F] matrix ---------------------
def test_matmul_chain_and_concat_order():
    w = wl.make_scoring("mm", 5, 4, [16, 8], 3, 5, 16 * wl.KIB, 64 * wl.MIB, 1.0, 64.0, False, "f32", 5)
    m = oracle_model(w)
    X = orc.materialise_inputs(m, w.dyn, w.scal, w.part, w.cred)
    S, C, F = X.shape
    assert (S, C, F) == (5, 15, 4 * 3 + 4 + 2) and F == w.F
    # column order: layer-major / stat-minor block, scalars, partition, credit
    assert X[2, 7, 1 * 3 + 2] == pytest.approx(_phi(float(w.dyn[2, 1, 2]), w.stat_enc[2]), rel=1e-13)
    assert X[2, 7, 12 + 1] == pytest.approx(_phi(float(w.scal[2, 1]), w.scal_enc[1]), rel=1e-13)
    assert X[2, 7, F - 2] == pytest.approx(_phi(float(w.part[7 // 5]), w.part_enc), rel=1e-13)
    assert X[2, 7, F - 1] == pytest.approx(_phi(float(w.cred[7 % 5]), w.cred_enc), rel=1e-13, abs=1e-15)
    h = X.reshape(S * C, F)
    for k in range(2):
        h = np.maximum(h @ m.W[k].T + m.b[k], 0.0)
    ref = (h @ m.W[2].T + m.b[2]).reshape(S, C)
    got = orc.score(m, w.dyn, w.scal, w.part, w.cred)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_layer1_splits_into_scenario_and_candidate_terms():
    """W1 [x_s (+) cfg] = A[s] + B[c]: the identity a factorised implementation relies on."""
    w = wl.make_scoring("fact", 4, 3, [8], 3, 3, 16 * wl.KIB, 64 * wl.MIB, 1.0, 8.0, True, "f32", 9)
    m = oracle_model(w)
    X = orc.materialise_inputs(m, w.dyn, w.scal, w.part, w.cred)
    Fs = w.F - 2
    A = X[:, 0, :Fs] @ m.W[0][:, :Fs].T
    Bt = X[0, :, Fs:] @ m.W[0][:, Fs:].T + m.b[0]
    full = X @ m.W[0].T + m.b[0]
    np.testing.assert_allclose(full, A[:, None, :] + Bt[None, :, :], rtol=0, atol=1e-12)


# ---- closed form of a network with no hidden layer -----------------------------------------------
@pytest.mark.parametrize("wp,wc", [(0.7, 0.3), (-0.7, 0.3), (0.7, -0.3), (-0.2, -0.9)])
def test_linear_net_picks_grid_corner(wp, wc):
    w = wl.make_scoring("lin", 6, 5, [], 4, 5, 16 * wl.KIB, 64 * wl.MIB, 1.0, 64.0, False, "f32", 11)
    W = [w.W[0].astype(np.float64).copy()]
    W[0][0, -2], W[0][0, -1] = wp, wc
    m = oracle_model(w, W=W)
    sc = orc.score(m, w.dyn, w.scal, w.part, w.cred)
    idx, best, _ = orc.select(sc)
    p = 3 if wp > 0 else 0
    q = 4 if wc > 0 else 0
    assert (idx == p * 5 + q).all()       # same corner for every scenario: phi is monotone
    # closed-form value: w_s.x_s + wp*phi(S_p) + wc*phi(S_c) + b
    X = orc.materialise_inputs(m, w.dyn, w.scal, w.part, w.cred)
    ref = X[:, p * 5 + q, :] @ W[0][0] + float(w.b[0][0])
    np.testing.assert_allclose(best, ref, rtol=1e-12)
    # phi at the grid ends is -/+ sqrt(3) for the log-centred transform
    assert X[0, 0, -2] == pytest.approx(-math.sqrt(3.0), rel=1e-6)
    assert X[0, -1, -2] == pytest.approx(math.sqrt(3.0), rel=1e-6)


def test_all_ties_pick_index_zero():
    w = wl.make_scoring("tie", 3, 2, [], 3, 3, 16 * wl.KIB, 64 * wl.MIB, 1.0, 8.0, True, "f32", 12)
    W = [w.W[0].astype(np.float64).copy()]
    W[0][0, -2:] = 0.0
    sc = orc.score(oracle_model(w, W=W), w.dyn, w.scal, w.part, w.cred)
    assert (sc == sc[:, :1]).all()
    idx, _, second = orc.select(sc)
    assert (idx == 0).all() and (second == sc[:, 0]).all()


# ---- invariants of the selection ----------------------------------------------------------------------
def test_candidate_permutation_invariance():
    w = wl.make_scoring("perm", 7, 4, [12, 6], 4, 6, 16 * wl.KIB, 64 * wl.MIB, 1.0, 64.0, False, "f32", 13)
    m = oracle_model(w)
    base = orc.score(m, w.dyn, w.scal, w.part, w.cred)
    rng = np.random.default_rng(0)
    pp, pq = rng.permutation(4), rng.permutation(6)
    perm = orc.score(m, w.dyn, w.scal, w.part[pp], w.cred[pq])
    # scores are the same numbers, moved (bit for bit: each candidate is evaluated on its own)
    assert (perm.reshape(7, 4, 6) == base.reshape(7, 4, 6)[:, pp][:, :, pq]).all()
    i0, b0, _ = orc.select(base)
    i1, b1, _ = orc.select(perm)
    assert (b0 == b1).all()
    assert (w.part[i0 // 6] == w.part[pp][i1 // 6]).all()
    assert (w.cred[i0 % 6] == w.cred[pq][i1 % 6]).all()


def test_monotone_output_transform_keeps_choice():
    w = wl.make_scoring("mono", 9, 4, [10], 5, 5, 16 * wl.KIB, 64 * wl.MIB, 1.0, 64.0, False, "f32", 14)
    i0, _, _ = orc.select(orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred))
    W = [x.astype(np.float64) for x in w.W]
    b = [x.astype(np.float64) for x in w.b]
    W[-1] = 4.0 * W[-1]
    b[-1] = 4.0 * b[-1] + 7.0
    i1, _, _ = orc.select(orc.score(oracle_model(w, W=W, b=b), w.dyn, w.scal, w.part, w.cred))
    assert (i0 == i1).all()


# ---- the transform ----------------------------------------------------------------------------------------
def test_encode_spot_values():
    enc_bytes = wl._log_uniform_enc(4 * wl.KIB, 400 * wl.MIB)
    assert orc.encode_value(4 * wl.KIB, enc_bytes) == pytest.approx(-math.sqrt(3.0), rel=1e-12)
    assert orc.encode_value(400 * wl.MIB, enc_bytes) == pytest.approx(math.sqrt(3.0), rel=1e-12)
    assert orc.encode_value(math.sqrt(4 * wl.KIB * 400 * wl.MIB), enc_bytes) == pytest.approx(0.0, abs=1e-12)
    assert orc.encode_value(2.0, wl._time_enc()) == pytest.approx(0.0, abs=1e-15)
    assert orc.encode_value(2.0 * math.e, wl._time_enc()) == pytest.approx(2.0, rel=1e-12)
    assert orc.encode_value(50.5, (0, 50.5, 0.1)) == 0.0
    assert orc.encode_value(60.5, (0, 50.5, 0.1)) == pytest.approx(1.0, rel=1e-12)


def test_encoded_inputs_are_standardised():
    """The transform constants make every non-one-hot column roughly zero-mean / unit-variance."""
    w = wl.make_config(2, S=512)
    m = oracle_model(w)
    Xs = orc.materialise_inputs(m, w.dyn, w.scal, w.part[:1], w.cred[:1])[:, 0, :]
    cols = [c for c in range(w.F - 2) if c not in (w.L * 3 + 2, w.L * 3 + 3)]
    mean, std = Xs[:, cols].mean(axis=0), Xs[:, cols].std(axis=0)
    assert np.abs(mean).max() < 0.25 and np.abs(std - 1.0).max() < 0.25


# ---- selection edge cases --------------------------------------------------------------------------------
def test_select_nan_inf_and_stride():
    sc = np.array([[np.nan, 1.0, np.nan, 1.0, 0.5, 99.0],
                   [np.nan, np.nan, np.nan, np.nan, np.nan, 99.0],
                   [-np.inf, np.inf, 3.0, np.inf, 0.0, 99.0],
                   [-np.inf, -np.inf, -np.inf, -np.inf, -np.inf, 99.0]])
    idx, best, second = orc.select(sc[:, :5].copy())
    assert list(idx) == [1, -1, 1, 0]
    assert best[0] == 1.0 and math.isnan(best[1]) and best[2] == np.inf and best[3] == -np.inf
    assert second[0] == 1.0 and second[2] == np.inf
    # strided rows: the 6th column is padding that must be ignored
    lib_idx = np.empty(4, dtype=np.int32)
    import ctypes as C
    b = np.empty(4)
    s2 = np.empty(4)
    rc = orc._load().orc_select(np.ascontiguousarray(sc).ctypes.data_as(orc._dp), C.c_int64(4), C.c_int(5),
                                C.c_int64(6), lib_idx.ctypes.data_as(C.POINTER(C.c_int32)),
                                b.ctypes.data_as(orc._dp), s2.ctypes.data_as(orc._dp))
    assert rc == 0 and list(lib_idx) == [1, -1, 1, 0]


def test_select_matches_numpy_argmax_on_random_rows():
    rng = np.random.default_rng(3)
    sc = rng.standard_normal((200, 37))
    sc[rng.random(sc.shape) < 0.2] = 0.25                                   # plenty of exact ties
    sc[:20] = np.minimum(sc[:20], 0.25)                                     # ... also at the top
    idx, best, second = orc.select(sc)
    assert (idx == np.argmax(sc, axis=1)).all()          # numpy: first occurrence on ties
    assert (best == sc.max(axis=1)).all()
    assert (second == np.sort(sc, axis=1)[:, -2]).all()


# ---- tensor-encoder pooling ---------------------------------------------------------------------------
def test_tensor_pooling_is_permutation_invariant_and_a_mean():
    w = wl.make_tensor_encoder("te", 3, [6], [4, 5], 2, 3, "f32", 21, n_blocks=3, per_block=2, extra=2)
    m = oracle_model(w)
    base = orc.score(m, w.dyn, w.scal, w.part, w.cred)
    perm = np.random.default_rng(1).permutation(w.L)
    np.testing.assert_allclose(orc.score(m, w.dyn[:, perm], w.scal, w.part, w.cred), base, rtol=1e-12, atol=1e-14)
    # one tensor repeated L times pools to that tensor's embedding: equals the L = 1 model
    rep = np.repeat(w.dyn[:, :1], w.L, axis=1)
    one = orc.Model(1, w.K, m.stat_enc, m.scal_enc, m.part_enc, m.cred_enc, m.hidden, m.W, m.b, m.te_W, m.te_b)
    np.testing.assert_allclose(orc.score(m, rep, w.scal, w.part, w.cred),
                               orc.score(one, w.dyn[:, :1], w.scal, w.part, w.cred), rtol=1e-12, atol=1e-14)
    # pooled block is the arithmetic mean of per-tensor embeddings (library ops)
    X = orc.materialise_inputs(m, w.dyn, w.scal, w.part, w.cred)
    t = np.stack([[_phi(float(w.dyn[s, l, k]), w.stat_enc[k]) for k in range(w.K)]
                  for s in range(3) for l in range(w.L)]).reshape(3, w.L, w.K)
    h = np.maximum(t @ m.te_W[0].T.astype(np.float64) + m.te_b[0], 0)
    h = np.maximum(h @ m.te_W[1].T.astype(np.float64) + m.te_b[1], 0)
    np.testing.assert_allclose(X[:, 0, :5], h.mean(axis=1), rtol=1e-12, atol=1e-14)


# ---- the diagnostic rounding mode (used by the GPU tests to tell kernel bugs from rounding noise) ----------
def test_diagnostic_rounding_is_the_bfloat16_format_rounding():
    import torch
    # the format: 8 significand bits, ties to even -- spot values from the definition
    assert orc.round_bf16_value(1.0) == 1.0
    assert orc.round_bf16_value(1.0 + 2.0 ** -8) == 1.0                      # tie -> even (1.0)
    assert orc.round_bf16_value(1.0 + 2.0 ** -7 + 2.0 ** -8) == 1.0 + 2.0 ** -6   # tie -> even (upwards)
    assert orc.round_bf16_value(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert orc.round_bf16_value(-3.0e38) == -float(torch.tensor(-3.0e38).bfloat16().float().abs())
    assert math.isnan(orc.round_bf16_value(float("nan"))) and orc.round_bf16_value(0.0) == 0.0
    # a library conversion on random values over many binades
    rng = np.random.default_rng(5)
    v = (rng.standard_normal(4000) * np.exp(rng.uniform(-60, 60, 4000))).astype(np.float32)
    want = torch.from_numpy(v).bfloat16().float().numpy()
    got = np.array([orc.round_bf16_value(float(x)) for x in v], dtype=np.float32)
    assert (got == want).all()


def test_diagnostic_rounding_is_a_no_op_on_exactly_representable_activations():
    """Small-integer inputs, weights and biases: every stored value is an integer below 256, which bfloat16
    holds exactly, so the rounding mode must reproduce the plain oracle bit for bit; with generic weights it
    must differ, but by no more than a few roundings of 2^-9 relative size."""
    rng = np.random.default_rng(9)
    S, L, K, P, Q = 4, 3, 2, 3, 2
    lin = (0, 0.0, 1.0)
    hidden = [5, 4, 3]
    dims = [L * K + 1 + 2] + hidden + [1]
    W = [rng.integers(-1, 2, (dims[i + 1], dims[i])).astype(np.float32) for i in range(len(dims) - 1)]
    b = [rng.integers(-2, 3, dims[i + 1]).astype(np.float32) for i in range(len(dims) - 1)]
    dyn = rng.integers(0, 3, (S, L, K)).astype(np.float32)
    scal = rng.integers(0, 3, (S, 1)).astype(np.float32)
    part, cred = np.array([1, 2, 3], np.float32), np.array([0, 1], np.float32)
    m = orc.Model(L, K, [lin] * K, [lin], lin, lin, hidden, W, b)
    plain = orc.score(m, dyn, scal, part, cred)
    assert np.abs(plain).max() > 0
    m.round_stored_bf16 = True
    assert (orc.score(m, dyn, scal, part, cred) == plain).all()
    # generic weights: rounding shows, and stays small
    w = wl.make_scoring("rnd", 6, 4, [32, 32], 3, 3, 16 * wl.KIB, 64 * wl.MIB, 1.0, 8.0, False, "bf16", 31)
    mg = oracle_model(w)
    exact = orc.score(mg, w.dyn, w.scal, w.part, w.cred)
    mg.round_stored_bf16 = True
    rounded = orc.score(mg, w.dyn, w.scal, w.part, w.cred)
    d = np.abs(rounded - exact).max() / np.abs(exact).max()
    assert 0 < d < 2e-2


def test_integer_network_equals_integer_arithmetic():
    """On an integer-valued network the oracle's fp64 result must equal the same network evaluated in int64
    (a different arithmetic altogether), for every scenario and candidate; with the tensor encoder the pooled
    block is a multiple of 1/2, so twice the score is compared."""
    w = wl.make_integer_scoring("int", 5, 7, [48, 32, 16], 4, 5, "f32", 77, nonzeros=16)
    ref = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
    Wi = [x.astype(np.int64) for x in w.W]
    bi = [x.astype(np.int64) for x in w.b]
    for s in range(5):
        for p in range(4):
            for q in range(5):
                x = np.concatenate([w.dyn[s].reshape(-1), w.scal[s], [w.part[p]], [w.cred[q]]]).astype(np.int64)
                for k in range(3):
                    x = np.maximum(Wi[k] @ x + bi[k], 0)
                assert ref[s, p * 5 + q] == float((Wi[3] @ x + bi[3])[0])
    t = wl.make_integer_tensor_encoder("int-te", 4, 6, [64, 64], 3, 3, "bf16", 78)
    ref = orc.score(oracle_model(t), t.dyn, t.scal, t.part, t.cred)
    Wi = [x.astype(np.int64) for x in t.W]
    bi = [x.astype(np.int64) for x in t.b]
    A, a, Bm, bb = (t.te_W[0].astype(np.int64), t.te_b[0].astype(np.int64), t.te_W[1].astype(np.int64),
                    t.te_b[1].astype(np.int64))
    for s in range(4):
        e = sum(np.maximum(Bm @ np.maximum(A @ t.dyn[s, l].astype(np.int64) + a, 0) + bb, 0) for l in range(6))
        assert (e % 3 == 0).all()                    # six tensors of two kinds: the sum is a multiple of three
        pool2 = e // 3                               # = 2 * mean
        for p in range(3):
            for q in range(3):
                # everything doubled: x2 = 2x, biases doubled, relu commutes with the positive factor
                x2 = np.concatenate([pool2, 2 * t.scal[s].astype(np.int64), [2 * int(t.part[p])], [2 * int(t.cred[q])]])
                for k in range(2):
                    x2 = np.maximum(Wi[k] @ x2 + 2 * bi[k], 0)
                assert 2.0 * ref[s, p * 3 + q] == float((Wi[2] @ x2 + 2 * bi[2])[0])
