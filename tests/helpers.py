"""Glue used by the tests: turn a drawn workload into the oracle's model description."""
import numpy as np

from oracle import oracle as orc


def oracle_model(wl, W=None, b=None) -> orc.Model:
    return orc.Model(L=wl.L, K=wl.K, stat_enc=list(wl.stat_enc), scal_enc=list(wl.scal_enc),
                     part_enc=wl.part_enc, cred_enc=wl.cred_enc, hidden=list(wl.hidden),
                     W=[np.asarray(w, dtype=np.float64) for w in (W if W is not None else wl.W)],
                     b=[np.asarray(x, dtype=np.float64) for x in (b if b is not None else wl.b)],
                     te_W=getattr(wl, "te_W", None), te_b=getattr(wl, "te_b", None), te_kind=getattr(wl, "te_kind", "mlp"),
                     loss_kind=getattr(wl, "loss_kind", "mse"))


# ---- parity measures -----------------------------------------------------------------------
def score_scale(ref):
    """Per-scenario yardstick for score errors: the larger of the scenario's own score magnitude
    max_c |ref[s, c]| and the root-mean-square of all oracle scores of the batch.

    Scores are zero-mean (random weights), so element-wise relative error is unbounded, and even a
    whole scenario's scores can sit near zero by cancellation while the activations that produced
    them are O(1); a reduced-precision pipeline's error follows the activations, not the cancelled
    sum.  The batch RMS is the natural unit of "one score" and floors the per-scenario scale."""
    ref = np.asarray(ref, dtype=np.float64)
    finite = ref[np.isfinite(ref)]
    rms = float(np.sqrt(np.mean(finite ** 2))) if finite.size else 1.0
    with np.errstate(invalid="ignore"):
        scale = np.nanmax(np.where(np.isfinite(ref), np.abs(ref), np.nan), axis=1) \
            if np.isfinite(ref).any(axis=1).all() else \
            np.array([np.abs(r[np.isfinite(r)]).max() if np.isfinite(r).any() else 0.0 for r in ref])
    scale = np.maximum(scale, rms)
    return np.where(scale > 0, scale, 1.0)


def scaled_error(got, ref):
    """max over scenarios and candidates of |got - ref| / score_scale(ref)[s]."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return float((np.abs(got - ref) / score_scale(ref)[:, None]).max())


def tensor_scaled_error(got, ref):
    """||got - ref||_inf / ||ref||_inf over the whole score matrix (the per-tensor norm also used for
    gradients and weights)."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max() if ref.size else 1.0
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0)) if ref.size else 0.0


def check_selection(got_idx, ref_scores, tol, per_scenario=True):
    """Index must equal the oracle's wherever the oracle's top-2 margin, relative to the score
    yardstick (per scenario, or the matrix-wide maximum magnitude), exceeds ``tol``; elsewhere the
    chosen candidate's oracle score must be within tol * scale of the top.  Returns the fraction
    of scenarios where the exact check applied."""
    ref_scores = np.asarray(ref_scores, dtype=np.float64)
    ridx, rbest, rsecond = orc.select(ref_scores)
    if per_scenario:
        scale = score_scale(ref_scores)
    else:
        den = np.abs(ref_scores).max()
        scale = np.full(ref_scores.shape[0], den if den > 0 else 1.0)
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


def frob_error(got, ref):
    """||got - ref||_F / ||ref||_F."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / (den if den > 0 else 1.0))


def full_size_sample(S, n_first, n_last, n_mid, edge, seed):
    """Scenario indices for an oracle sample of a full-size run (see ``workloads.sample_scenarios``)."""
    from paper_2112_13509_amd import workloads as wl
    return wl.sample_scenarios(S, n_first, n_last, n_mid, edge, seed)


def check_against_matched(got, refq, tolq):
    """The GPU's scores against the oracle in its rounding-matched mode, strict per-scenario measure.
    What is left between the two is accumulation order, which now and then lands a pre-activation on the
    other side of a bf16 rounding boundary; in wide, deep scorers such a flip perturbs every unit of the
    next layer a little and so causes further flips there.  Single scenarios are hit, and the worst of a
    sample grows with its size; so: at least 95 % of the scenarios within ``tolq`` and every one within twice
    that.  Returns (worst scenario's error, fraction of scenarios above tolq)."""
    got, refq = np.asarray(got, dtype=np.float64), np.asarray(refq, dtype=np.float64)
    per_scenario = (np.abs(got - refq) / score_scale(refq)[:, None]).max(axis=1)
    worst, above = float(per_scenario.max()), float((per_scenario > tolq).mean())
    assert worst <= 2 * tolq, (worst, tolq)
    assert above <= 0.05, (above, tolq)
    return worst, above
