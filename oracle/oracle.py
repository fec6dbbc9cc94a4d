"""ctypes front-end of the fp64 CPU oracle (``autobyte_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the benchmark's CPU-baseline
leg.  It never touches the GPU library and shares nothing with it.  Arrays go in as NumPy arrays of
any float dtype and are widened to float64 exactly before the C code sees them.

Paper passages followed are cited in the C file next to each function (arXiv 2112.13509,
Table 1, Section 3.1 "Meta network architecture", Eq. 1, Eq. 2, Section 3.2).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "autobyte_oracle.c")
_LIB = os.path.join(_HERE, "liborc.so")

ENC_LINEAR, ENC_LOG = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def build_sanitized() -> str:
    """The same source compiled with AddressSanitizer and UndefinedBehaviorSanitizer (gcc, -O1), as
    ``liborc_san.so``; a process that loads it needs gcc's ASan runtime preloaded.  Returns the library path."""
    out = os.path.join(_HERE, "liborc_san.so")
    if not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        tmp = out + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, out)
    return out


def _load():
    global _lib
    if _lib is None:
        # AUTOBYTE_ORACLE_LIB: an already built variant of this library (the sanitizer run of the tests uses it)
        _lib = C.CDLL(os.environ.get("AUTOBYTE_ORACLE_LIB") or build())
        _lib.orc_encode_value.restype = C.c_double
        _lib.orc_encode_value.argtypes = [C.c_double, C.c_int, C.c_double, C.c_double]
        _lib.orc_round_bf16_value.restype = C.c_double
        _lib.orc_round_bf16_value.argtypes = [C.c_double]
        _lib.orc_num_threads.restype = C.c_int
    return _lib


_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int)
_dpp = C.POINTER(_dp)


class _CModel(C.Structure):
    _fields_ = [("L", C.c_int), ("K", C.c_int), ("Ns", C.c_int),
                ("stat_kind", _ip), ("stat_shift", _dp), ("stat_scale", _dp),
                ("scal_kind", _ip), ("scal_shift", _dp), ("scal_scale", _dp),
                ("cfg_kind", _ip), ("cfg_shift", _dp), ("cfg_scale", _dp),
                ("tensor_encoder", C.c_int), ("te_h0", C.c_int), ("te_h1", C.c_int),
                ("te_W", _dpp), ("te_b", _dpp),
                ("n_hidden", C.c_int), ("hidden", _ip),
                ("W", _dpp), ("b", _dpp), ("round_stored_bf16", C.c_int),
                ("n_out", C.c_int), ("loss_kind", C.c_int)]


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr_array(arrs: Sequence[np.ndarray]):
    pa = (_dp * max(1, len(arrs)))()
    for i, a in enumerate(arrs):
        pa[i] = a.ctypes.data_as(_dp) if a is not None else None
    return pa


@dataclass
class Model:
    """Plain description of one meta-network.  ``*_enc`` are lists of (kind, shift, scale)."""
    L: int
    K: int
    stat_enc: List[Tuple[int, float, float]]
    scal_enc: List[Tuple[int, float, float]]
    part_enc: Tuple[int, float, float]
    cred_enc: Tuple[int, float, float]
    hidden: List[int]
    W: List[np.ndarray]            # n_hidden + 1 matrices [out, in]
    b: List[np.ndarray]
    te_W: Optional[List[np.ndarray]] = None   # tensor encoder: [[h0,K],[h1,h0]] or None
    te_b: Optional[List[np.ndarray]] = None
    te_kind: str = "mlp"                     # "mlp": shared per-layer MLP + mean; "lstm": embedding + 2-layer LSTM,
                                             #   te_W = [[E,K], [4H,E+H], [4H,2H]], te_b = [[E], [4H], [4H]]
    round_stored_bf16: bool = False          # diagnostic: mimic a bf16 pipeline's stored activations
    loss_kind: str = "mse"                   # "mse": mean of the summed squared error; "l2norm": mean Euclidean norm (Eq. 2)
    _keep: list = field(default_factory=list, repr=False)

    @property
    def Ns(self) -> int:
        return len(self.scal_enc)

    @property
    def stats_width(self) -> int:
        if self.te_W is None:
            return self.L * self.K + self.Ns
        return (self.te_W[1].shape[0] // 4 if self.te_kind == "lstm" else self.te_W[1].shape[0]) + self.Ns

    @property
    def F(self) -> int:
        return self.stats_width + 2

    @property
    def n_out(self) -> int:
        """Entries of V (one per worker, Table 1); candidates are ranked by their mean."""
        return int(np.asarray(self.W[-1]).shape[0])

    def _c(self) -> _CModel:
        keep = []

        def enc_arrays(encs):
            kinds = np.ascontiguousarray([e[0] for e in encs] or [0], dtype=np.int32)
            sh = _f64([e[1] for e in encs] or [0.0])
            sc = _f64([e[2] for e in encs] or [1.0])
            keep.extend([kinds, sh, sc])
            return kinds.ctypes.data_as(_ip), sh.ctypes.data_as(_dp), sc.ctypes.data_as(_dp)

        m = _CModel()
        m.L, m.K, m.Ns = int(self.L), int(self.K), self.Ns
        assert len(self.stat_enc) == self.K
        m.stat_kind, m.stat_shift, m.stat_scale = enc_arrays(self.stat_enc)
        m.scal_kind, m.scal_shift, m.scal_scale = enc_arrays(self.scal_enc)
        m.cfg_kind, m.cfg_shift, m.cfg_scale = enc_arrays([self.part_enc, self.cred_enc])
        if self.te_W is not None:
            tw = [_f64(w) for w in self.te_W]
            tb = [_f64(x) for x in self.te_b]
            if self.te_kind == "lstm":
                E, H = tw[0].shape[0], tw[1].shape[0] // 4
                assert tw[0].shape == (E, self.K) and tw[1].shape == (4 * H, E + H) and tw[2].shape == (4 * H, 2 * H)
                assert tb[0].shape == (E,) and tb[1].shape == (4 * H,) and tb[2].shape == (4 * H,)
                m.tensor_encoder, m.te_h0, m.te_h1 = 2, E, H
            else:
                assert tw[0].shape[1] == self.K and tw[1].shape[1] == tw[0].shape[0]
                m.tensor_encoder, m.te_h0, m.te_h1 = 1, tw[0].shape[0], tw[1].shape[0]
            pw, pb = _ptr_array(tw), _ptr_array(tb)
            keep.extend(tw + tb + [pw, pb])
            m.te_W, m.te_b = C.cast(pw, _dpp), C.cast(pb, _dpp)
        else:
            m.tensor_encoder, m.te_h0, m.te_h1 = 0, 0, 0
        hid = np.ascontiguousarray(list(self.hidden) or [0], dtype=np.int32)
        m.n_hidden = len(self.hidden)
        m.hidden = hid.ctypes.data_as(_ip)
        Ws = [_f64(w) for w in self.W]
        bs = [_f64(x) for x in self.b]
        assert len(Ws) == len(self.hidden) + 1 == len(bs)
        widths = [self.F] + list(self.hidden) + [self.n_out]
        for k, w in enumerate(Ws):
            assert w.shape == (widths[k + 1], widths[k]), (k, w.shape, widths)
            assert bs[k].shape == (widths[k + 1],)
        pW, pb = _ptr_array(Ws), _ptr_array(bs)
        keep.extend([hid, pW, pb] + Ws + bs)
        m.W, m.b = C.cast(pW, _dpp), C.cast(pb, _dpp)
        m.round_stored_bf16 = 1 if self.round_stored_bf16 else 0
        m.n_out = self.n_out
        m.loss_kind = {"mse": 0, "l2norm": 1}[self.loss_kind]
        self._keep = keep
        return m


def encode_value(x: float, enc: Tuple[int, float, float]) -> float:
    return float(_load().orc_encode_value(float(x), int(enc[0]), float(enc[1]), float(enc[2])))


def round_bf16_value(x: float) -> float:
    """The rounding used by ``round_stored_bf16`` (diagnostic mode), for one value."""
    return float(_load().orc_round_bf16_value(float(x)))


def num_threads() -> int:
    return int(_load().orc_num_threads())


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError("oracle %s failed with code %d" % (what, rc))


def score(model: Model, dyn, scal, part, cred, layers_of=None) -> np.ndarray:
    """Predicted V for every scenario and candidate: returns float64 [S, P*Q], c = p*Q + q.
    ``layers_of`` [S] (encoder models only): how many of the L padded layers each scenario really has.
    ``part`` [P] and ``cred`` [Q] are shared by all scenarios; given as [S, P] and [S, Q] every scenario
    has its own grid."""
    lib = _load()
    dyn, scal, part, cred = _f64(dyn), _f64(scal), _f64(part), _f64(cred)
    S = dyn.shape[0]
    assert dyn.shape == (S, model.L, model.K) and scal.shape == (S, model.Ns)
    per_scenario = part.ndim == 2
    assert cred.ndim == part.ndim and (not per_scenario or (part.shape[0] == S and cred.shape[0] == S))
    P, Q = part.shape[-1], cred.shape[-1]
    out = np.empty((S, P * Q), dtype=np.float64)
    cm = model._c()
    lo = None if layers_of is None else np.ascontiguousarray(layers_of, dtype=np.int32)
    assert lo is None or lo.shape == (S,)
    _check(lib.orc_score_grids(C.byref(cm), dyn.ctypes.data_as(_dp), scal.ctypes.data_as(_dp),
                               C.c_int64(S), None if lo is None else lo.ctypes.data_as(_ip),
                               part.ctypes.data_as(_dp), C.c_int(P),
                               cred.ctypes.data_as(_dp), C.c_int(Q), C.c_int(1 if per_scenario else 0),
                               out.ctypes.data_as(_dp)), "score")
    return out


def predict_v(model: Model, dyn, scal, part, cred, cand, layers_of=None) -> np.ndarray:
    """The predicted speed vector V (one entry per output unit, Table 1) of candidate ``cand[s]`` = p*Q + q for
    every scenario: float64 [S, n_out]; NaN where cand[s] is not a valid candidate index."""
    lib = _load()
    dyn, scal, part, cred = _f64(dyn), _f64(scal), _f64(part), _f64(cred)
    S = dyn.shape[0]
    assert dyn.shape == (S, model.L, model.K) and scal.shape == (S, model.Ns)
    per_scenario = part.ndim == 2
    P, Q = part.shape[-1], cred.shape[-1]
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    assert cand.shape == (S,)
    out = np.empty((S, model.n_out), dtype=np.float64)
    cm = model._c()
    lo = None if layers_of is None else np.ascontiguousarray(layers_of, dtype=np.int32)
    _check(lib.orc_predict_v(C.byref(cm), dyn.ctypes.data_as(_dp), scal.ctypes.data_as(_dp), C.c_int64(S),
                             None if lo is None else lo.ctypes.data_as(_ip),
                             part.ctypes.data_as(_dp), C.c_int(P), cred.ctypes.data_as(_dp), C.c_int(Q),
                             C.c_int(1 if per_scenario else 0), cand.ctypes.data_as(_ip),
                             out.ctypes.data_as(_dp)), "predict_v")
    return out


def lstm_encode(model: Model, dyn, layers_of=None) -> np.ndarray:
    """The LSTM temporal encoder alone (Section 3.1): last hidden state of the second layer, float64 [S, H]."""
    lib = _load()
    dyn = _f64(dyn)
    S = dyn.shape[0]
    assert model.te_kind == "lstm" and dyn.shape == (S, model.L, model.K)
    out = np.empty((S, model.te_W[1].shape[0] // 4), dtype=np.float64)
    cm = model._c()
    lo = None if layers_of is None else np.ascontiguousarray(layers_of, dtype=np.int32)
    _check(lib.orc_lstm_encode(C.byref(cm), dyn.ctypes.data_as(_dp), C.c_int64(S),
                               None if lo is None else lo.ctypes.data_as(_ip), out.ctypes.data_as(_dp)),
           "lstm_encode")
    return out


def materialise_inputs(model: Model, dyn, scal, part, cred) -> np.ndarray:
    """The explicit input vectors, float64 [S, P*Q, F]."""
    lib = _load()
    dyn, scal, part, cred = _f64(dyn), _f64(scal), _f64(part), _f64(cred)
    S, P, Q = dyn.shape[0], part.shape[0], cred.shape[0]
    out = np.empty((S, P * Q, model.F), dtype=np.float64)
    cm = model._c()
    _check(lib.orc_materialise_inputs(C.byref(cm), dyn.ctypes.data_as(_dp), scal.ctypes.data_as(_dp),
                                      C.c_int64(S), part.ctypes.data_as(_dp), C.c_int(P),
                                      cred.ctypes.data_as(_dp), C.c_int(Q),
                                      out.ctypes.data_as(_dp)), "materialise_inputs")
    return out


def select(scores, row_stride: Optional[int] = None):
    """Per-row argmax (lowest index on ties, NaN never wins, -1 if all NaN).

    Returns (best_idx int32 [S], best_score float64 [S], runner_up float64 [S])."""
    lib = _load()
    scores = _f64(scores)
    S, Cn = scores.shape
    stride = Cn if row_stride is None else int(row_stride)
    idx = np.empty(S, dtype=np.int32)
    best = np.empty(S, dtype=np.float64)
    second = np.empty(S, dtype=np.float64)
    _check(lib.orc_select(scores.ctypes.data_as(_dp), C.c_int64(S), C.c_int(Cn), C.c_int64(stride),
                          idx.ctypes.data_as(C.POINTER(C.c_int32)), best.ctypes.data_as(_dp),
                          second.ctypes.data_as(_dp)), "select")
    return idx, best, second


def trigger(scores, cur_idx, observed=None, gain_threshold=0.05, error_threshold=0.10, row_stride=None):
    """Optimization Trigger on float32 scores [S, C]: returns (best_idx, gain, reconfigure, adapt)."""
    lib = _load()
    scores = np.ascontiguousarray(np.asarray(scores, dtype=np.float32))
    S, Cn = scores.shape
    stride = Cn if row_stride is None else int(row_stride)
    Cn = Cn if row_stride is None else Cn
    cur = np.ascontiguousarray(np.asarray(cur_idx, dtype=np.int32))
    obs = None if observed is None else np.ascontiguousarray(np.asarray(observed, dtype=np.float32))
    best = np.empty(S, dtype=np.int32)
    gain = np.empty(S, dtype=np.float32)
    reconf = np.empty(S, dtype=np.uint8)
    adapt = np.empty(S, dtype=np.uint8)
    fp = C.POINTER(C.c_float)
    _check(lib.orc_trigger(scores.ctypes.data_as(fp), C.c_int64(S), C.c_int(Cn), C.c_int64(stride),
                           cur.ctypes.data_as(C.POINTER(C.c_int32)),
                           obs.ctypes.data_as(fp) if obs is not None else None,
                           C.c_float(gain_threshold), C.c_float(error_threshold),
                           best.ctypes.data_as(C.POINTER(C.c_int32)), gain.ctypes.data_as(fp),
                           reconf.ctypes.data_as(C.POINTER(C.c_uint8)),
                           adapt.ctypes.data_as(C.POINTER(C.c_uint8))), "trigger")
    return best, gain, reconf.astype(bool), adapt.astype(bool)


@dataclass
class TrainState:
    """Master parameters and Adam moments (float64), updated in place by :func:`update`."""
    W: List[np.ndarray]
    b: List[np.ndarray]
    mW: List[np.ndarray]
    vW: List[np.ndarray]
    mb: List[np.ndarray]
    vb: List[np.ndarray]
    t: int = 0                      # number of steps taken so far

    @staticmethod
    def fresh(W, b) -> "TrainState":
        W = [_f64(w).copy() for w in W]
        b = [_f64(x).copy() for x in b]
        z = lambda xs: [np.zeros_like(x) for x in xs]
        return TrainState(W, b, z(W), z(W), z(b), z(b), 0)

    def copy(self) -> "TrainState":
        c = lambda xs: [x.copy() for x in xs]
        return TrainState(c(self.W), c(self.b), c(self.mW), c(self.vW), c(self.mb), c(self.vb), self.t)


def update(model: Model, state: TrainState, x_raw, target, lr=1e-3, beta1=0.9, beta2=0.999,
           eps=1e-8, do_adam=True, forward_weights=None, want_grads=True, first_trainable=0):
    """One online-adaptation step (forward, loss of ``model.loss_kind``, back-propagation, Adam) on ``state``.
    ``target`` is [B], or [B, n_out] when the output layer predicts one speed per worker.

    ``model`` supplies the feature layout and widths; its own W/b are ignored in favour of
    ``state``.  ``forward_weights`` optionally replaces the weights used by forward/backward
    (e.g. a bf16-rounded copy) while Adam still updates the fp64 masters.
    ``first_trainable`` > 0 is the transfer-learning form: scorer layers below it stay frozen.
    Returns dict(loss, gW, gb, yhat)."""
    lib = _load()
    x_raw, target = _f64(x_raw), _f64(target)
    B = x_raw.shape[0]
    n_out = int(state.W[-1].shape[0])
    assert model.te_W is None and x_raw.shape == (B, model.F)
    assert target.shape == (B, n_out) or (n_out == 1 and target.shape == (B,))
    tmp = Model(model.L, model.K, model.stat_enc, model.scal_enc, model.part_enc, model.cred_enc,
                model.hidden, state.W, state.b, loss_kind=model.loss_kind)
    tmp.round_stored_bf16 = model.round_stored_bf16
    cm = tmp._c()
    Wf = [_f64(w) for w in (forward_weights if forward_weights is not None else state.W)]
    n = len(state.W)
    gW = [np.zeros_like(w) for w in state.W] if want_grads else [None] * n
    gb = [np.zeros_like(x) for x in state.b] if want_grads else [None] * n
    yhat = np.empty((B, n_out) if target.ndim == 2 else B, dtype=np.float64)
    loss = C.c_double(0.0)
    for lst in (state.W, state.b, state.mW, state.vW, state.mb, state.vb):
        for a in lst:
            assert a.dtype == np.float64 and a.flags.c_contiguous
    t = state.t + 1
    _check(lib.orc_update_tail(C.byref(cm), x_raw.ctypes.data_as(_dp), target.ctypes.data_as(_dp),
                          C.c_int64(B), _ptr_array(Wf), _ptr_array(state.b),
                          _ptr_array(state.W), _ptr_array(state.b),
                          _ptr_array(state.mW), _ptr_array(state.vW),
                          _ptr_array(state.mb), _ptr_array(state.vb),
                          C.c_int64(t), C.c_double(lr), C.c_double(beta1), C.c_double(beta2),
                          C.c_double(eps), C.c_int(1 if do_adam else 0), C.byref(loss),
                          _ptr_array(gW), _ptr_array(gb), yhat.ctypes.data_as(_dp),
                          C.c_int(int(first_trainable))), "update")
    if do_adam:
        state.t = t
    return {"loss": float(loss.value), "gW": gW, "gb": gb, "yhat": yhat}


def replay_mix(x_new, t_new, x_old, t_old, pick):
    """Minibatch assembled from freshly observed rows and the offline set (Section 3.2: online
    adaptation refreshes the offline-trained model and extends its dataset with the new samples): entry i of ``pick`` >= 0 takes new row pick[i], entry < 0 takes
    old row -pick[i] - 1; an index outside its pool gives a NaN row.  Targets are [n] or [n, n_out] (one observed
    speed per worker).  Returns (x [B, F], target [B] or [B, n_out])."""
    x_new, t_new, x_old, t_old = _f64(x_new), _f64(t_new), _f64(x_old), _f64(t_old)
    pick = np.asarray(pick, dtype=np.int64)
    F = x_new.shape[1] if x_new.size else x_old.shape[1]
    t_ref = t_new if t_new.size else t_old
    x = np.full((pick.shape[0], F), np.nan)
    t = np.full((pick.shape[0],) + t_ref.shape[1:], np.nan)
    for i, p in enumerate(pick):
        if 0 <= p < x_new.shape[0]:
            x[i], t[i] = x_new[p], t_new[p]
        elif p < 0 and -p - 1 < x_old.shape[0]:
            x[i], t[i] = x_old[-p - 1], t_old[-p - 1]
    return x, t
