"""GPU parity of the temporal encoder (embedding + two-layer LSTM over the layer sequence, Section 3.1 "Meta
network architecture") inside ab_score_candidates, against the fp64 oracle."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2112_13509_amd import workloads as wl
from helpers import oracle_model, scaled_error, tensor_scaled_error, check_selection, check_against_matched

pytestmark = pytest.mark.gpu

TOL_MATCHED = 1e-2  # against the oracle rounding its stored values to bf16 where the kernels do (strict measure;
                    # 95 % of the scenarios within it, all within twice that: see helpers.check_against_matched)
TOL = 2e-2          # bf16 bar, per-tensor norm (the recurrent state is rounded to bf16 once per step and layer)


def compare(w, scores, idx, best, label=""):
    m = oracle_model(w)
    ref = orc.score(m, w.dyn, w.scal, w.part, w.cred)
    err, strict = tensor_scaled_error(scores, ref), scaled_error(scores, ref)
    active = check_selection(idx, ref, TOL)
    m.round_stored_bf16 = True
    errq, _ = check_against_matched(scores, orc.score(m, w.dyn, w.scal, w.part, w.cred), TOL_MATCHED)
    msg = "%s L=%d S=%d: rel err %.3g (tol %g), strict %.3g, vs rounding-matched oracle %.3g, exact-index check on %.0f%%" % (
        label, w.L, w.S, err, TOL, strict, errq, 100 * active)
    print(msg)
    assert err <= TOL and strict <= 5e-2, msg
    rows = np.arange(w.S)
    assert (idx >= 0).all() and np.array_equal(best, scores[rows, idx])
    assert np.array_equal(idx, np.argmax(scores, axis=1))


def test_lstm_encoder_small_and_ragged():
    from gpu_helpers import Scorer
    # L = 1 (one step), 17 and 33 (chunks of 16 steps plus a tail), 50; S = 1, 5, 33, 70 (blocks of 32 plus a tail)
    for (nb, per, extra), S in (((1, 1, 0), 1), ((2, 8, 1), 5), ((2, 16, 1), 33), ((3, 16, 2), 70)):
        w = wl.make_lstm_encoder("lstm-small", S, [64, 64], 3, 3, "bf16", 77 + S, n_blocks=nb, per_block=per, extra=extra)
        compare(w, *Scorer(w).run(), label="small")


def test_lstm_encoder_alone_through_a_probe_scorer():
    """Scorer reduced to a probe: the first hidden layer copies encoder outputs (+ and -) and the output unit
    sums them with weights, so an error of the encoder shows up undiluted."""
    from gpu_helpers import Scorer
    w = wl.make_lstm_encoder("lstm-probe", 40, [128], 2, 2, "bf16", 5, n_blocks=4, per_block=16, extra=3)
    H = 64
    W0 = np.zeros_like(w.W[0])
    W0[np.arange(H), np.arange(H)] = 1.0
    W0[H + np.arange(H), np.arange(H)] = -1.0
    w.W[0], w.b[0] = W0, np.zeros_like(w.b[0])
    rng = np.random.default_rng(1)
    wo = wl.bf16_round(rng.standard_normal(H).astype(np.float32))
    w.W[1] = np.concatenate([wo, -wo])[None, :].astype(np.float32)          # sum_j wo[j] * h[j]
    w.b[1] = np.zeros_like(w.b[1])
    scores, idx, best = Scorer(w).run()
    enc = orc.lstm_encode(oracle_model(w), w.dyn)
    want = enc @ wo.astype(np.float64)
    got = scores[:, 0]
    assert np.abs(scores - scores[:, :1]).max() == 0.0                     # the grid does not enter
    err = np.abs(got - want).max() / np.abs(want).max()
    print("encoder probe: max err %.3g of max |value| %.3g" % (err, np.abs(want).max()))
    assert err <= TOL


def test_lstm_encoder_full_length_sampled():
    from gpu_helpers import Scorer
    w = wl.make_config(6, S=96)
    assert w.L == 400
    compare(w, *Scorer(w).run(), label="cfg6 subset")


def test_lstm_encoder_nan_statistic_poisons_only_its_scenario():
    from gpu_helpers import Scorer
    w = wl.make_lstm_encoder("lstm-nan", 40, [64, 64], 3, 3, "bf16", 9, n_blocks=2, per_block=8, extra=0)
    w.dyn[7, 3, 1] = np.nan
    scores, idx, best = Scorer(w).run()
    assert np.isnan(scores[7]).all() and idx[7] == -1
    ok = np.arange(40) != 7
    ref = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
    assert np.isfinite(scores[ok]).all()
    assert tensor_scaled_error(scores[ok], ref[ok]) <= TOL


@pytest.mark.parametrize("kind", ["mlp", "lstm"])
def test_scenarios_with_fewer_layers_than_the_padded_tensor(kind):
    """Per-scenario layer counts: mean over / recurrence through a scenario's own layers only; whatever sits in
    the padding (NaN here) must not reach the result."""
    from gpu_helpers import Scorer
    S = 70
    if kind == "mlp":
        w = wl.make_tensor_encoder("te-len", S, [64, 64], [128, 128], 3, 3, "bf16", 41, n_blocks=3, per_block=16, extra=2)
    else:
        w = wl.make_lstm_encoder("lstm-len", S, [64, 64], 3, 3, "bf16", 41, n_blocks=3, per_block=16, extra=2)
    rng = np.random.default_rng(8)
    lens = rng.integers(1, w.L + 1, S).astype(np.int32)
    lens[:4] = [1, w.L, 17, 33]
    for s in range(S):
        w.dyn[s, lens[s]:] = np.nan
    scores, idx, best = Scorer(w).run(layers_of=lens)
    ref = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred, layers_of=lens)
    assert np.isfinite(scores).all() and np.isfinite(ref).all()
    err, strict = tensor_scaled_error(scores, ref), scaled_error(scores, ref)
    print("%s with own layer counts: rel err %.3g strict %.3g" % (kind, err, strict))
    assert err <= TOL and strict <= 5e-2
    check_selection(idx, ref, TOL)
    # out-of-range counts are clamped to [1, L]
    lens2 = lens.copy()
    lens2[lens == w.L] = w.L + 50
    lens2[lens == 1] = -3
    s2, _, _ = Scorer(w).run(layers_of=lens2)
    assert np.array_equal(s2, scores)


def test_integer_tensor_encoder_with_own_layer_counts_is_reproduced_exactly():
    """The exact case behind the mean-pooled encoder with every scenario having its own (even) number of layers:
    two kinds of tensor take turns, so the mean over any even prefix is a multiple of 1/2 and nothing rounds;
    scores and choices must equal the oracle's bit for bit (the padding holds NaN)."""
    from gpu_helpers import Scorer
    S, L = 90, 48
    w = wl.make_integer_tensor_encoder("int-te-len", S, L, [256, 256], 8, 8, "bf16", 4100, alternate=True)
    lens = (2 * np.random.default_rng(3).integers(1, L // 2 + 1, S)).astype(np.int32)
    lens[:3] = [2, L, 34]
    for s in range(S):
        w.dyn[s, lens[s]:] = np.nan
    m = oracle_model(w)
    ref = orc.score(m, w.dyn, w.scal, w.part, w.cred, layers_of=lens)
    m.round_stored_bf16 = True
    assert (orc.score(m, w.dyn, w.scal, w.part, w.cred, layers_of=lens) == ref).all()
    scores, idx, best = Scorer(w).run(layers_of=lens)
    ridx, rbest, _ = orc.select(ref)
    assert np.isfinite(ref).all() and len(np.unique(ref)) > 8
    assert (scores == ref.astype(np.float32)).all()
    assert (idx == ridx).all() and (best == rbest.astype(np.float32)).all()
