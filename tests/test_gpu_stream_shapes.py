"""Shapes that walk the streaming hidden-layer GEMMs through their corner cases (tile counts that do not divide
evenly over the work-groups, ragged last row tile, one or two K slabs per tile, column-tile counts that do not
divide the work-groups of an XCD), each against the fp64 oracle."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2112_13509_amd import binding as ab
from paper_2112_13509_amd import workloads as wl
from helpers import oracle_model, scaled_error, tensor_scaled_error, check_selection

pytestmark = pytest.mark.gpu


def run_and_compare(w, label):
    from gpu_helpers import Scorer
    names = []
    ab.ab_set_trace(lambda kernel, phase, work, is_bytes: names.append(kernel) if phase == 0 else None)
    try:
        scores, idx, best = Scorer(w).run()
    finally:
        ab.ab_set_trace(None)
    ref = orc.score(oracle_model(w), w.dyn, w.scal, w.part, w.cred)
    err, strict = tensor_scaled_error(scores, ref), scaled_error(scores, ref)
    print("%s: S=%d C=%d hidden=%s launches=%s rel err %.3g strict %.3g" % (
        label, w.S, w.C, w.hidden, sorted(set(n for n in names if n.startswith("gemm_hidden"))), err, strict))
    assert err <= 2e-2 and strict <= 5e-2
    check_selection(idx, ref, 2e-2)
    assert np.array_equal(idx, np.argmax(scores, axis=1)) and np.array_equal(best, scores[np.arange(w.S), idx])


# The 256 x 256 kernels take a hidden GEMM from 64 tiles per launch on; every case below has at least that many.
@pytest.mark.parametrize("S,P,Q,hidden,label", [
    (600, 16, 16, [256, 256], "600 row tiles over 256 work-groups (2 or 3 each), generated operand + fused output"),
    (257, 16, 16, [256, 256, 256], "257 row tiles: one work-group walks two tiles, the others one"),
    (205, 20, 16, [256, 256, 256], "C = 320: stored-operand layer with a ragged last row tile (65600 rows)"),
    (90, 16, 16, [256, 768, 256], "three column tiles (do not divide the 32 work-groups of an XCD), K = 768"),
    (260, 16, 16, [128, 256, 256], "K = 128: two slabs per tile in the first hidden GEMM"),
    (260, 16, 16, [64, 256, 256], "K = 64: the first hidden GEMM falls back to the one-tile-per-work-group kernel"),
    (70, 32, 32, [1024, 1024], "1024 candidates: four row tiles per scenario"),
    (300, 16, 16, [256, 256, 64, 256], "K = 64 in a stored-operand layer: one slab per tile"),
    (40, 16, 16, [256, 1280, 256], "five column tiles in a stored layer: bias through the scalar cache, K = 1280 after it"),
    (40, 16, 16, [256, 256, 1280], "five column tiles in the layer that feeds the output unit"),
    (40, 16, 16, [1280, 1280], "five column tiles, generated operand with K = 1280 (one tile per work-group) feeding the output unit"),
    (150, 16, 16, [512, 1024, 512], "four and two column tiles: bias and output weights in registers, tiles change column block"),
    (32, 16, 16, [4096, 4096], "the widest layers the library takes: sixteen column tiles, K = 4096 (64 slabs per tile)"),
])
def test_streaming_gemm_corner_shapes(S, P, Q, hidden, label):
    w = wl.make_scoring("stream-shapes", S, 16, hidden, P, Q, 16 * wl.KIB, 64 * wl.MIB, 1.0, 64.0, False, "bf16",
                        1000 + S + len(hidden))
    run_and_compare(w, label)
