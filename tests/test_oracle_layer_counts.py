"""Pins for scenarios with fewer layers than the padded statistics tensor holds (Section 3.1 "Meta network
architecture": jobs differ in their number of layers and are embedded into a fixed-width feature space): a scenario
with n layers must score exactly like the same model declared with L = n on the truncated statistics."""
import dataclasses

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2112_13509_amd import workloads as wl
from helpers import oracle_model


def _truncated(m, n):
    return dataclasses.replace(m, L=n, _keep=[])


@pytest.mark.parametrize("kind", ["mlp", "lstm"])
def test_fewer_layers_equal_a_shorter_model(kind):
    if kind == "mlp":
        w = wl.make_tensor_encoder("te-len", 6, [64, 64], [128, 128], 3, 3, "bf16", 5, n_blocks=2, per_block=5, extra=2)
    else:
        w = wl.make_lstm_encoder("lstm-len", 6, [64, 64], 3, 3, "bf16", 5, n_blocks=2, per_block=5, extra=2)
    m = oracle_model(w)
    lens = np.array([12, 1, 7, 12, 3, 9], dtype=np.int32)
    got = orc.score(m, w.dyn, w.scal, w.part, w.cred, layers_of=lens)
    garbage = w.dyn.copy()
    for s, n in enumerate(lens):
        ref = orc.score(_truncated(m, int(n)), w.dyn[s:s + 1, :n], w.scal[s:s + 1], w.part, w.cred)
        assert np.array_equal(got[s], ref[0]), (kind, s)
        garbage[s, n:] = np.nan                                    # what lies past a scenario's layers is never read
    assert np.array_equal(orc.score(m, garbage, w.scal, w.part, w.cred, layers_of=lens), got)
    assert np.array_equal(orc.score(m, w.dyn, w.scal, w.part, w.cred, layers_of=np.full(6, 12, np.int32)),
                          orc.score(m, w.dyn, w.scal, w.part, w.cred))
    # out-of-range counts are clamped to [1, L]
    assert np.array_equal(orc.score(m, w.dyn, w.scal, w.part, w.cred, layers_of=np.array([0, -5, 99, 12, 1, 1], np.int32)),
                          orc.score(m, w.dyn, w.scal, w.part, w.cred, layers_of=np.array([1, 1, 12, 12, 1, 1], np.int32)))
    if kind == "lstm":
        enc = orc.lstm_encode(m, w.dyn, layers_of=lens)
        for s, n in enumerate(lens):
            assert np.array_equal(enc[s], orc.lstm_encode(_truncated(m, int(n)), w.dyn[s:s + 1, :n])[0])


def test_flat_layout_refuses_layer_counts():
    w = wl.make_config(1, S=2)
    with pytest.raises(Exception):
        orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred, layers_of=np.array([1, 1], np.int32))
