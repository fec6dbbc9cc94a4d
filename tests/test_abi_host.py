"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments with the documented status before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2112_13509_amd import binding as ab
from paper_2112_13509_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ab.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    return ab.load()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "autobyte.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(ab_[a-z_]+)\s*\(", header))
    assert {"ab_score_candidates", "ab_select_best", "ab_online_update", "ab_workspace_bytes",
            "ab_status_string", "ab_version", "ab_trigger", "ab_set_trace", "ab_online_update_tail",
            "ab_replay_mix", "ab_score_candidates_static", "ab_static_scratch_bytes"} <= names
    for n in names:
        assert hasattr(lib, n), n
    assert ab.ab_version() >= 100
    assert ab.ab_status_string(0) == "ok" and "NULL" in ab.ab_status_string(-1)


def test_struct_layout_matches_header_sizes():
    # ab_enc = 12 bytes; desc = 3 ints + 58 encs (16 + 40 + 2) + int + 8 ints + int + 2 ints + int + 2 ints
    assert C.sizeof(ab.ab_enc) == 12
    assert C.sizeof(ab.ab_model_desc) == 4 * 3 + 12 * (16 + 40 + 2) + 4 + 4 * 8 + 4 + 8 + 4 + 8
    assert C.sizeof(ab.ab_params) == 8 * (12 * 7 + 1)
    assert C.sizeof(ab.ab_stats) == 32 and C.sizeof(ab.ab_grid) == 32


def _desc(cfg=2):
    return ab.desc_from_workload(wl.make_config(cfg, S=1))


def test_workspace_bytes(lib):
    d = _desc(3)
    small, big = ab.ab_workspace_bytes(d, 16, 256), ab.ab_workspace_bytes(d, 65536, 256)
    assert 0 < small < big
    # cfg3 at full size: scenario rows + two ping-pong activation chunks of 2^20 rows x 1024 bf16
    assert 2 * (1 << 20) * 1024 * 2 < big < 6 * (1 << 30)
    assert ab.ab_workspace_bytes(d, 0, 0, 0) == 0
    d.compute_dtype = 7
    assert ab.ab_workspace_bytes(d, 16, 256) == 0
    du = ab.desc_from_workload(wl.make_update(N=64, batch=64, L=2, hidden=(64,)))
    assert ab.ab_workspace_bytes(du, 0, 0, 64) > 0


def test_encoder_options_in_the_descriptor(lib):
    # the temporal encoder (embedding + two-layer LSTM): widths {32, 64}, bf16 only, three parameter layers in front
    w = wl.make_lstm_encoder("lstm-host", 2, [64, 64], 2, 2, "bf16", 1, n_blocks=1, per_block=2, extra=0)
    d = ab.desc_from_workload(w)
    assert d.tensor_encoder == 2 and list(d.enc_hidden) == [32, 64]
    assert ab.ab_workspace_bytes(d, 16, 4) > 0
    p = _fake_params(3 + 2)                                   # the output layer's pointers are missing
    assert _call_score(lib, d, params=p) == -1
    # per-scenario layer counts: encoders only, 4-byte aligned
    assert _call_score(lib, d, params=_fake_params(6), stats=ab.ab_stats(0x3000, 0x4000, 4, 0x7002)) == -4
    flat = _desc(1)
    assert _call_score(lib, flat, params=_fake_params(3), stats=ab.ab_stats(0x3000, 0x4000, 4, 0x7000)) == -6
    d.enc_hidden[1] = 128
    assert ab.ab_workspace_bytes(d, 16, 4) == 0 and _call_score(lib, d, params=_fake_params(6)) == -6
    d.enc_hidden[1] = 64
    d.compute_dtype = 0
    assert _call_score(lib, d, params=_fake_params(6)) == -6
    d.compute_dtype = 1
    d.tensor_encoder = 3
    assert _call_score(lib, d, params=_fake_params(6)) == -2


def _call_score(lib, d, params=None, stats=None, grid=None, scores=0x1000, idx=0x2000, best=None,
                ws=0x100000, ws_bytes=1 << 40):
    p = params or ab.ab_params()
    st = stats or ab.ab_stats(0x3000, 0x4000, 4)
    gr = grid or ab.ab_grid(0x5000, 2, 0x6000, 2)
    return lib.ab_score_candidates(C.byref(d), C.byref(p), C.byref(st), C.byref(gr), scores, idx, best,
                                   ws, ws_bytes, None)


def _fake_params(n):
    p = ab.ab_params()
    for k in range(n):
        p.W[k] = 0x10000 * (k + 1)
        p.b[k] = 0x10000 * (k + 1) + 0x8000
    return p


def test_score_argument_errors(lib):
    d = _desc(2)
    p = _fake_params(3)
    assert lib.ab_score_candidates(None, None, None, None, None, None, None, None, 0, None) == -1
    assert _call_score(lib, d, p, scores=None, idx=None) == -1                 # no output requested
    assert _call_score(lib, d, p, idx=None, best=0x7000) == -1                 # best_score without best_idx
    assert _call_score(lib, d, ab.ab_params()) == -1                           # weights missing
    assert _call_score(lib, d, p, grid=ab.ab_grid(0x5000, 0, 0x6000, 2)) == -2  # empty grid
    assert _call_score(lib, d, p, stats=ab.ab_stats(0x3000, 0x4000, -1)) == -2
    assert _call_score(lib, d, p, ws=None) == -5
    assert _call_score(lib, d, p, ws_bytes=16) == -5
    assert _call_score(lib, d, p, ws=0x100010) == -4                           # workspace not 256-aligned
    bad = _fake_params(3)
    bad.W[1] = 0x20004
    assert _call_score(lib, d, bad) == -4                                      # weight not 16-aligned
    d2 = _desc(2)
    d2.compute_dtype = 5
    assert _call_score(lib, d2, p) == -3
    d3 = _desc(2)
    d3.hidden[0] = 100
    assert _call_score(lib, d3, p) == -6                                       # width not a multiple of 64
    d4 = _desc(2)
    d4.n_hidden = 0                                                            # no hidden layer: the linear scorer
    assert ab.ab_workspace_bytes(d4, 16, 4) == 256                             # (one launch, no workspace of its own)
    assert _call_score(lib, d4, ab.ab_params()) == -1                          # its one weight matrix is missing
    d4.tensor_encoder = 1
    d4.enc_hidden[0] = d4.enc_hidden[1] = 128
    assert _call_score(lib, d4, p) == -6 and ab.ab_workspace_bytes(d4, 16, 4) == 0   # ... takes flat statistics only
    d5 = _desc(2)
    d5.n_stats = 99
    assert _call_score(lib, d5, p) == -2
    d6 = _desc(2)
    d6.n_outputs = 17                                                          # more entries of V than the ABI holds
    assert _call_score(lib, d6, p) == -2 and ab.ab_workspace_bytes(d6, 16, 4) == 0
    d6.n_outputs, d6.loss_kind = 8, 2                                          # unknown loss
    assert _call_score(lib, d6, p) == -2
    # S = 0 is a valid no-op that never touches the device
    assert _call_score(lib, d, p, stats=ab.ab_stats(None, None, 0)) == 0
    assert _call_score(lib, d, p, stats=ab.ab_stats(None, None, 0), scores=None, idx=None, ws=None) == 0


def test_select_and_update_argument_errors(lib):
    assert lib.ab_select_best(None, 4, 4, 4, 0x1000, None, None) == -1
    assert lib.ab_select_best(0x1000, 4, 4, 4, None, None, None) == -1
    assert lib.ab_select_best(0x1000, 4, 0, 4, 0x2000, None, None) == -2
    assert lib.ab_select_best(0x1000, 4, 8, 4, 0x2000, None, None) == -2       # stride < C
    assert lib.ab_select_best(0x1002, 4, 4, 4, 0x2000, None, None) == -4
    assert lib.ab_select_best(0x1000, 0, 4, 4, 0x2000, None, None) == 0
    f = C.c_float
    trig = lambda sc=0x1000, S=4, Cn=4, st=4, cur=0x2000, obs=0x3000, best=0x4000, gain=None, rec=0x5000, ad=None: \
        lib.ab_trigger(sc, S, Cn, st, cur, obs, f(0.05), f(0.1), best, gain, rec, ad, None)
    assert trig(sc=None) == -1 and trig(cur=None) == -1 and trig(best=None) == -1 and trig(rec=None) == -1
    assert trig(obs=None, ad=0x6000) == -1                                     # adapt needs observations
    assert trig(Cn=0) == -2 and trig(Cn=8, st=4) == -2 and trig(S=-1) == -2
    assert trig(sc=0x1001) == -4
    assert trig(S=0) == 0
    u = wl.make_update(N=64, batch=64, L=2, hidden=(64,))
    d = ab.desc_from_workload(u)
    p = ab.ab_params()
    call = lambda prm, x=0x1000, y=0x2000, B=64, ws=0x100000, n=1 << 40: lib.ab_online_update(
        C.byref(d), C.byref(prm), x, y, B, f(1e-3), f(0.9), f(0.999), f(1e-8), None, ws, n, None)
    assert call(p) == -1
    full = ab.ab_params()
    for k in range(2):
        for name in ("W", "b", "W_master", "adam_mW", "adam_vW", "adam_mb", "adam_vb"):
            getattr(full, name)[k] = 0x100000 * (k + 1)
    full.step = 0x900000
    assert call(full, x=None) == -1
    assert call(full, B=0) == -2
    assert call(full, ws=None) == -5
    assert call(full, n=10) == -5
    # a first layer of 2^32 weights or more is refused (the Adam launch numbers a tensor's elements with 32 bits)
    wide = ab.make_desc(1 << 16, 16, [(0, 0.0, 1.0)] * 16, [], (1, 12.0, 0.5), (1, 2.0, 0.5), (4096,), "bf16")
    assert lib.ab_online_update(C.byref(wide), C.byref(full), 0x1000, 0x2000, 64, f(1e-3), f(0.9), f(0.999),
                                f(1e-8), None, 0x100000, 1 << 60, None) == -6
    dte = ab.desc_from_workload(wl.make_config(5, S=1))
    assert lib.ab_online_update(C.byref(dte), C.byref(full), 0x1000, 0x2000, 64, f(1e-3), f(0.9), f(0.999),
                                f(1e-8), None, 0x100000, 1 << 40, None) == -6


def test_transfer_learning_argument_errors(lib):
    f = C.c_float
    u = wl.make_update(N=64, batch=64, L=2, hidden=(64, 64))
    d = ab.desc_from_workload(u)
    p = ab.ab_params()
    tail = lambda k0, B=64, prm=p: lib.ab_online_update_tail(C.byref(d), C.byref(prm), 0x1000, 0x2000, B, k0, f(1e-3), f(0.9),
                                                             f(0.999), f(1e-8), None, 0x100000, 1 << 40, None)
    assert tail(-1) == -2 and tail(3) == -2 and tail(0, B=0) == -2
    assert tail(2) == -1                                       # parameter pointers missing
    # frozen layers need W and b only
    q = ab.ab_params()
    for k in range(3):
        q.W[k], q.b[k] = 0x10000 * (k + 1), 0x10000 * (k + 1) + 0x8000
    q.step = 0x90000
    assert tail(2, prm=q) == -1                                # the output layer's master copy and moments are missing
    q.W_master[2] = q.adam_mW[2] = q.adam_vW[2] = q.adam_mb[2] = q.adam_vb[2] = 0xa0000
    assert lib.ab_online_update_tail(C.byref(d), C.byref(q), 0x1000, 0x2000, 64, 2, f(1e-3), f(0.9), f(0.999), f(1e-8),
                                     None, 0x100000, 16, None) == -5     # everything present: the workspace is too small
    mix = lambda xn=0x1000, tn=0x2000, nn=4, xo=0x3000, to=0x4000, no=4, pick=0x5000, B=8, F=6, xout=0x6000, tout=0x7000, n_out=1: \
        lib.ab_replay_mix(xn, tn, nn, xo, to, no, pick, B, F, n_out, xout, tout, None)
    assert mix(F=0) == -2 and mix(nn=-1) == -2 and mix(B=-1) == -2
    assert mix(n_out=0) == -2 and mix(n_out=17) == -2
    assert mix(pick=None) == -1 and mix(xout=None) == -1 and mix(xn=None) == -1 and mix(to=None) == -1
    assert mix(xout=0x6001) == -4
    assert mix(B=0) == 0


def test_binding_refuses_cpu_tensors(lib):
    import torch
    w = wl.make_config(1)
    d = ab.desc_from_workload(w)
    with pytest.raises(TypeError):
        ab.ab_select_best(torch.zeros(2, 4), torch.zeros(2, dtype=torch.int32))


def test_static_scratch_form_checks_its_arguments_on_the_host(lib):
    """The allocation-free scoring entry point refuses bad arguments and oversized problems before any
    device call is made (so these run without a GPU)."""
    assert ab.ab_static_scratch_bytes() == 32 << 20
    d = ab.make_desc(128, 3, [(1, 0.7, 2.0)] * 3, [(0, 0.0, 1.0)] * 4, (1, 12.0, 0.5), (1, 2.0, 0.5),
                     (1024, 1024, 1024, 1024), "bf16")
    call = lambda desc, prm, st, gr: lib.ab_score_candidates_static(
        None if desc is None else C.byref(desc), None if prm is None else C.byref(prm),
        None if st is None else C.byref(st), None if gr is None else C.byref(gr), 0x7000, 0x8000, None, None)
    p = ab.ab_params()
    assert call(None, p, ab.ab_stats(0x3000, 0x4000, 4), ab.ab_grid(0x5000, 16, 0x6000, 16)) == -1
    assert call(d, None, ab.ab_stats(0x3000, 0x4000, 4), ab.ab_grid(0x5000, 16, 0x6000, 16)) == -1
    big = ab.ab_stats(0x3000, 0x4000, 4096)
    assert ab.ab_workspace_bytes(d, 4096, 256) > ab.ab_static_scratch_bytes()
    assert call(d, p, big, ab.ab_grid(0x5000, 16, 0x6000, 16)) == -5
    bad = ab.make_desc(128, 3, [(1, 0.7, 2.0)] * 3, [(0, 0.0, 1.0)] * 4, (1, 12.0, 0.5), (1, 2.0, 0.5),
                       (1000,), "bf16")
    assert call(bad, p, ab.ab_stats(0x3000, 0x4000, 4), ab.ab_grid(0x5000, 16, 0x6000, 16)) == -6


def test_statistics_per_layer_limits(lib):
    """Sixteen statistics per layer (one backward time per worker of a sixteen-worker job, Table 1) are taken by
    the flat layout; the two encoders take eight and refuse more."""
    enc = [(1, 0.7, 2.0)] * 16
    flat = ab.make_desc(4, 16, enc, [(0, 0.0, 1.0)] * 38, (1, 12.0, 0.5), (1, 2.0, 0.5), (64, 64), "bf16")
    assert ab.ab_workspace_bytes(flat, 8, 16) > 0
    with pytest.raises(ValueError):
        ab.make_desc(4, 17, enc + [(1, 0.7, 2.0)], [], (1, 12.0, 0.5), (1, 2.0, 0.5), (64,), "bf16")
    flat.n_stats = 17
    assert ab.ab_workspace_bytes(flat, 8, 16) == 0
    for kind in ("mlp", "lstm"):
        te = ab.make_desc(4, 9, enc[:9], [(0, 0.0, 1.0)] * 2, (1, 12.0, 0.5), (1, 2.0, 0.5), (64, 64), "bf16",
                          te_hidden=(128, 128) if kind == "mlp" else (32, 64), te_kind=kind)
        assert ab.ab_workspace_bytes(te, 8, 16) == 0
        assert _call_score(lib, te, params=_fake_params(6)) == -6
        te.n_stats = 8
        assert ab.ab_workspace_bytes(te, 8, 16) > 0


def test_prediction_vector_form_checks_its_arguments(lib):
    w = wl.make_config(1)
    d = ab.desc_from_workload(w)
    p = _fake_params(3)
    call = lambda idx, v: lib.ab_score_candidates_v(C.byref(d), C.byref(p), C.byref(ab.ab_stats(0x3000, 0x4000, 4)),
                                                    C.byref(ab.ab_grid(0x5000, 2, 0x6000, 2)), 0x7000, idx, None, v,
                                                    0x100000, 1 << 40, None)
    assert call(None, 0x9000) == -1            # the vector is that of the chosen candidate: needs best_idx
    assert call(0x8000, 0x9002) == -4
