"""How far bf16 storage alone moves the results, measured on the oracle itself (CPU only).

The GPU path keeps activations in bf16 wherever it stores them, as the bf16 configurations demand.
The oracle has a diagnostic mode that rounds its stored values at the same places and changes nothing
else (fp64 accumulation, same order of steps).  The distance between the oracle's two modes is
therefore what any bf16 pipeline must be expected to show against the exact oracle; the tolerances of
the GPU parity tests lean on the figures asserted here:

* scores of the deep 1024-wide scorer (390 -> 1024^4 -> 1): within 1e-2 of the exact oracle in the
  per-tensor norm ||d||_inf / ||o||_inf, but already 1.7e-2 away in the strict per-scenario measure on
  a sample of 48 scenarios; that maximum grows with the sample (the GPU tests compute the same figure
  on their own, larger samples and hold the GPU to a small multiple of it), so 2e-2 in the strict
  measure is not a bar a bf16 pipeline can be held to, while 2e-2 in the per-tensor norm is;
* gradients: a unit whose pre-activation lies within the rounding noise of zero flips its ReLU mask,
  which makes that delta entry wrong by 100 %; a fraction f of flipped entries gives a relative
  Frobenius error of about sqrt(f), so the first layer's weight gradient is 2e-2 ... 6e-2 away at
  configuration 4's real shape although no entry is off by more than 2e-2 of the largest one.
"""
import numpy as np

from oracle import oracle as orc
from paper_2112_13509_amd import workloads as wl
from helpers import (oracle_model, scaled_error, tensor_scaled_error, check_selection, tensor_error,
                     frob_error)


def _both_modes(w):
    m = oracle_model(w)
    ref = orc.score(m, w.dyn, w.scal, w.part, w.cred)
    m.round_stored_bf16 = True
    return ref, orc.score(m, w.dyn, w.scal, w.part, w.cred)


def test_rounding_alone_on_the_deep_scorer_exceeds_the_strict_measure_but_not_the_tensor_norm():
    w = wl.make_config(3, S=48)                                     # 390 -> 1024^4 -> 1, 256 candidates
    ref, rounded = _both_modes(w)
    per_tensor, strict = tensor_scaled_error(rounded, ref), scaled_error(rounded, ref)
    print("cfg3 scorer, 48 scenarios: rounding alone moves scores by %.3g (per-tensor norm), %.3g (strict "
          "per-scenario measure)" % (per_tensor, strict))
    assert 3e-3 <= per_tensor <= 1.2e-2
    assert 1.2e-2 <= strict <= 3e-2
    # the selection rule of the parity tests holds for a pipeline that only rounds, and is not vacuous:
    # per-scenario scale, exact index wherever the exact oracle's top-2 margin exceeds 2e-2
    active = check_selection(orc.select(rounded)[0], ref, 2e-2, per_scenario=True)
    print("   exact-index rule (per-scenario scale, 2e-2) active on %.1f%% of scenarios" % (100 * active))
    assert active > 0


def test_rounding_alone_on_the_two_layer_scorers_stays_well_inside():
    for cfg, S in ((5, 12),):
        w = wl.make_config(cfg, S=S)
        ref, rounded = _both_modes(w)
        strict = scaled_error(rounded, ref)
        print("cfg%d scorer: rounding alone %.3g (strict)" % (cfg, strict))
        assert strict <= 1.5e-2


def test_rounding_alone_moves_first_layer_gradients_by_more_than_2e_2_in_the_frobenius_norm():
    u = wl.make_update()                                            # configuration 4's real shape
    st = orc.TrainState.fresh(u.W, u.b)
    rows = u.batch_indices(0)
    fw = [wl.bf16_round(w.astype(np.float32)).astype(np.float64) for w in st.W]
    mq = oracle_model(u)
    mq.round_stored_bf16 = True
    rounded = orc.update(mq, st.copy(), u.x_raw[rows], u.target[rows], forward_weights=fw, do_adam=False)
    ref = orc.update(oracle_model(u), st.copy(), u.x_raw[rows], u.target[rows], forward_weights=fw, do_adam=False)
    inf = [tensor_error(a, b) for a, b in zip(rounded["gW"] + rounded["gb"], ref["gW"] + ref["gb"])]
    fro = [frob_error(a, b) for a, b in zip(rounded["gW"] + rounded["gb"], ref["gW"] + ref["gb"])]
    print("cfg4 step 1, rounding alone: inf-norm errors %s" % ["%.2g" % e for e in inf])
    print("                             Frobenius errors %s" % ["%.2g" % e for e in fro])
    assert max(inf) <= 2e-2                       # the bound the GPU is held to at this shape
    assert 2e-2 < fro[0] <= 6e-2                  # first layer's weight gradient: mask flips
    assert max(fro[1:]) <= 1e-2
    assert abs(rounded["loss"] - ref["loss"]) <= 2e-3 * ref["loss"]
