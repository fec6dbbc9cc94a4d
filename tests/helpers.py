"""Glue used by the tests: turn a drawn workload into the oracle's model description."""
import numpy as np

from oracle import oracle as orc


def oracle_model(wl, W=None, b=None) -> orc.Model:
    return orc.Model(L=wl.L, K=wl.K, stat_enc=list(wl.stat_enc), scal_enc=list(wl.scal_enc),
                     part_enc=wl.part_enc, cred_enc=wl.cred_enc, hidden=list(wl.hidden),
                     W=[np.asarray(w, dtype=np.float64) for w in (W if W is not None else wl.W)],
                     b=[np.asarray(x, dtype=np.float64) for x in (b if b is not None else wl.b)],
                     te_W=getattr(wl, "te_W", None), te_b=getattr(wl, "te_b", None))
