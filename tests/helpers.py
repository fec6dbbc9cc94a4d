"""Glue used by the tests: turn a drawn workload into the oracle's model description."""
import numpy as np

from oracle import oracle as orc


def oracle_model(wl, W=None, b=None) -> orc.Model:
    return orc.Model(L=wl.L, K=wl.K, stat_enc=list(wl.stat_enc), scal_enc=list(wl.scal_enc),
                     part_enc=wl.part_enc, cred_enc=wl.cred_enc, hidden=list(wl.hidden),
                     W=[np.asarray(w, dtype=np.float64) for w in (W if W is not None else wl.W)],
                     b=[np.asarray(x, dtype=np.float64) for x in (b if b is not None else wl.b)],
                     te_W=getattr(wl, "te_W", None), te_b=getattr(wl, "te_b", None))


# ---- parity measures -----------------------------------------------------------------------
def scaled_error(got, ref):
    """max over scenarios and candidates of |got - ref| / scale_s with scale_s = max_c |ref[s, c]|.
    Scores of one scenario are zero-mean-ish, so element-wise relative error is unbounded; the
    scenario's own score magnitude is the yardstick instead."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max(axis=1, keepdims=True)
    scale = np.where(scale > 0, scale, 1.0)
    return float((np.abs(got - ref) / scale).max())


def check_selection(got_idx, ref_scores, tol):
    """Index must equal the oracle's wherever the oracle's top-2 margin (relative to the scenario's
    score magnitude) exceeds ``tol``; elsewhere the chosen candidate's oracle score must be within
    tol * scale of the top.  Returns the fraction of scenarios where the exact check applied."""
    ref_scores = np.asarray(ref_scores, dtype=np.float64)
    ridx, rbest, rsecond = orc.select(ref_scores)
    scale = np.abs(ref_scores).max(axis=1)
    scale = np.where(scale > 0, scale, 1.0)
    got_idx = np.asarray(got_idx)
    margin = (rbest - rsecond) / scale
    exact = margin > tol
    assert (got_idx[exact] == ridx[exact]).all(), "argmax differs where the oracle's margin exceeds tol"
    loose = ~exact
    if loose.any():
        rows = np.nonzero(loose)[0]
        assert (got_idx[rows] >= 0).all()
        chosen = ref_scores[rows, got_idx[rows]]
        assert (rbest[rows] - chosen <= tol * scale[rows]).all(), "chosen candidate is not near-optimal"
    return float(exact.mean())


def tensor_error(got, ref):
    """||got - ref||_inf / ||ref||_inf for gradients, moments and weights."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))
