"""Thin ctypes binding of ``libautobyte.so`` (see ``include/autobyte.h``).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch is
used for device memory and streams.  There is no fallback: if the library is missing, or a tensor
is not a contiguous ROCm tensor of the expected dtype, the call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import torch

AB_F32, AB_BF16 = 0, 1
AB_ENC_LINEAR, AB_ENC_LOG = 0, 1
AB_MAX_STATS, AB_MAX_SCALARS, AB_MAX_HIDDEN, AB_MAX_LAYERS = 16, 40, 8, 12

# AUTOBYTE_LIB: an already built variant of the library (the host-sanitizer run of the argument-check tests uses it)
_LIB_PATH = os.environ.get("AUTOBYTE_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libautobyte.so")
_lib = None


class ab_enc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("shift", C.c_float), ("scale", C.c_float)]


class ab_model_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_stats", C.c_int32), ("n_scalars", C.c_int32),
                ("enc_stat", ab_enc * AB_MAX_STATS), ("enc_scalar", ab_enc * AB_MAX_SCALARS),
                ("enc_partition", ab_enc), ("enc_credit", ab_enc),
                ("n_hidden", C.c_int32), ("hidden", C.c_int32 * AB_MAX_HIDDEN),
                ("tensor_encoder", C.c_int32), ("enc_hidden", C.c_int32 * 2),
                ("compute_dtype", C.c_int32), ("n_outputs", C.c_int32), ("loss_kind", C.c_int32)]


_vp = C.c_void_p


class ab_params(C.Structure):
    _fields_ = [("W", _vp * AB_MAX_LAYERS), ("b", _vp * AB_MAX_LAYERS),
                ("W_master", _vp * AB_MAX_LAYERS),
                ("adam_mW", _vp * AB_MAX_LAYERS), ("adam_vW", _vp * AB_MAX_LAYERS),
                ("adam_mb", _vp * AB_MAX_LAYERS), ("adam_vb", _vp * AB_MAX_LAYERS),
                ("step", _vp)]


class ab_stats(C.Structure):
    _fields_ = [("dyn", _vp), ("scalars", _vp), ("S", C.c_int64), ("layers_of", _vp)]


class ab_grid(C.Structure):
    _fields_ = [("partition_bytes", _vp), ("P", C.c_int32), ("credit_mult", _vp), ("Q", C.c_int32),
                ("per_scenario", C.c_int32)]


class AutoByteError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, ab_status_string(status), status))


def library_path() -> str:
    return _LIB_PATH


def load():
    """Load the HIP library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libautobyte.so is missing: run `python paper_2112_13509_amd/build.py` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        lib = C.CDLL(_LIB_PATH)
        lib.ab_version.restype = C.c_int32
        lib.ab_status_string.restype = C.c_char_p
        lib.ab_status_string.argtypes = [C.c_int32]
        lib.ab_workspace_bytes.restype = C.c_size_t
        lib.ab_workspace_bytes.argtypes = [C.POINTER(ab_model_desc), C.c_int64, C.c_int32, C.c_int64]
        lib.ab_score_candidates.restype = C.c_int32
        lib.ab_score_candidates.argtypes = [C.POINTER(ab_model_desc), C.POINTER(ab_params),
                                            C.POINTER(ab_stats), C.POINTER(ab_grid),
                                            _vp, _vp, _vp, _vp, C.c_size_t, _vp]
        lib.ab_score_candidates_v.restype = C.c_int32
        lib.ab_score_candidates_v.argtypes = [C.POINTER(ab_model_desc), C.POINTER(ab_params),
                                              C.POINTER(ab_stats), C.POINTER(ab_grid),
                                              _vp, _vp, _vp, _vp, _vp, C.c_size_t, _vp]
        lib.ab_static_scratch_bytes.restype = C.c_size_t
        lib.ab_static_scratch_bytes.argtypes = []
        lib.ab_score_candidates_static.restype = C.c_int32
        lib.ab_score_candidates_static.argtypes = [C.POINTER(ab_model_desc), C.POINTER(ab_params),
                                                   C.POINTER(ab_stats), C.POINTER(ab_grid),
                                                   _vp, _vp, _vp, _vp]
        lib.ab_select_best.restype = C.c_int32
        lib.ab_select_best.argtypes = [_vp, C.c_int64, C.c_int32, C.c_int64, _vp, _vp, _vp]
        lib.ab_trigger.restype = C.c_int32
        lib.ab_trigger.argtypes = [_vp, C.c_int64, C.c_int32, C.c_int64, _vp, _vp, C.c_float, C.c_float,
                                   _vp, _vp, _vp, _vp, _vp]
        lib.ab_online_update.restype = C.c_int32
        lib.ab_online_update.argtypes = [C.POINTER(ab_model_desc), C.POINTER(ab_params), _vp, _vp,
                                         C.c_int64, C.c_float, C.c_float, C.c_float, C.c_float,
                                         _vp, _vp, C.c_size_t, _vp]
        lib.ab_online_update_tail.restype = C.c_int32
        lib.ab_online_update_tail.argtypes = [C.POINTER(ab_model_desc), C.POINTER(ab_params), _vp, _vp,
                                              C.c_int64, C.c_int32, C.c_float, C.c_float, C.c_float, C.c_float,
                                              _vp, _vp, C.c_size_t, _vp]
        lib.ab_replay_mix.restype = C.c_int32
        lib.ab_replay_mix.argtypes = [_vp, _vp, C.c_int64, _vp, _vp, C.c_int64, _vp, C.c_int64, C.c_int32, C.c_int32,
                                      _vp, _vp, _vp]
        _lib = lib
    return _lib


TRACE_FN = C.CFUNCTYPE(None, C.c_char_p, C.c_int32, C.c_double, C.c_int32, C.c_void_p, C.c_void_p)
_trace_keepalive = None


def ab_set_trace(fn) -> None:
    """Install ``fn(kernel: str, phase: int, work: float, work_is_bytes: bool)`` around every kernel
    launch of the entry points (phase 0 before, 1 after), or switch tracing off with ``None``."""
    global _trace_keepalive
    lib = load()
    lib.ab_set_trace.restype = None
    lib.ab_set_trace.argtypes = [C.c_void_p, C.c_void_p]
    if fn is None:
        lib.ab_set_trace(None, None)
        _trace_keepalive = None
        return
    cb = TRACE_FN(lambda name, phase, work, is_bytes, stream, user: fn(name.decode(), phase, work, bool(is_bytes)))
    lib.ab_set_trace(C.cast(cb, C.c_void_p), None)
    _trace_keepalive = cb


class KernelTimer:
    """Device time of every traced launch, from events recorded on the current stream."""

    def __init__(self):
        self.records = []      # (kernel, work, is_bytes, start_event, end_event)
        self._open = None

    def __call__(self, name, phase, work, is_bytes):
        ev = torch.cuda.Event(enable_timing=True)
        ev.record(torch.cuda.current_stream())
        if phase == 0:
            self._open = (name, work, is_bytes, ev)
        else:
            n, w, b, start = self._open
            self.records.append((n, w, b, start, ev))

    def __enter__(self):
        ab_set_trace(self)
        return self

    def __exit__(self, *exc):
        ab_set_trace(None)

    def summary(self):
        """{kernel: dict(launches, total_ms, avg_ms, work, is_bytes)} after a device sync."""
        torch.cuda.synchronize()
        out = {}
        for n, w, b, s, e in self.records:
            d = out.setdefault(n, {"launches": 0, "total_ms": 0.0, "work": 0.0, "is_bytes": b})
            d["launches"] += 1
            d["total_ms"] += s.elapsed_time(e)
            d["work"] += w
        for d in out.values():
            d["avg_ms"] = d["total_ms"] / d["launches"]
        return out


def ab_version() -> int:
    return int(load().ab_version())


def ab_status_string(status: int) -> str:
    return load().ab_status_string(int(status)).decode()


# ---------------------------------------------------------------------------------------------
# building the plain-data arguments
# ---------------------------------------------------------------------------------------------
def make_desc(L: int, K: int, stat_enc: Sequence[Tuple[int, float, float]],
              scal_enc: Sequence[Tuple[int, float, float]], part_enc, cred_enc,
              hidden: Sequence[int], dtype: str, te_hidden: Optional[Sequence[int]] = None,
              te_kind: str = "mlp", n_outputs: int = 1, loss_kind: str = "mse") -> ab_model_desc:
    d = ab_model_desc()
    d.n_layers, d.n_stats, d.n_scalars = int(L), int(K), len(scal_enc)
    if K > AB_MAX_STATS or len(scal_enc) > AB_MAX_SCALARS or len(hidden) > AB_MAX_HIDDEN:
        raise ValueError("description exceeds the ABI's fixed array sizes")
    for i, e in enumerate(stat_enc):
        d.enc_stat[i] = ab_enc(int(e[0]), float(e[1]), float(e[2]))
    for i, e in enumerate(scal_enc):
        d.enc_scalar[i] = ab_enc(int(e[0]), float(e[1]), float(e[2]))
    d.enc_partition = ab_enc(int(part_enc[0]), float(part_enc[1]), float(part_enc[2]))
    d.enc_credit = ab_enc(int(cred_enc[0]), float(cred_enc[1]), float(cred_enc[2]))
    d.n_hidden = len(hidden)
    for i, h in enumerate(hidden):
        d.hidden[i] = int(h)
    d.tensor_encoder = (2 if te_kind == "lstm" else 1) if te_hidden else 0
    if te_hidden:
        d.enc_hidden[0], d.enc_hidden[1] = int(te_hidden[0]), int(te_hidden[1])
    d.compute_dtype = {"f32": AB_F32, "bf16": AB_BF16}[dtype]
    d.n_outputs = int(n_outputs)
    d.loss_kind = {"mse": 0, "l2norm": 1}[loss_kind]
    return d


def desc_from_workload(wl) -> ab_model_desc:
    return make_desc(wl.L, wl.K, wl.stat_enc, wl.scal_enc, wl.part_enc, wl.cred_enc, wl.hidden,
                     wl.dtype, getattr(wl, "te_hidden", None), getattr(wl, "te_kind", "mlp"),
                     n_outputs=int(wl.W[-1].shape[0]), loss_kind=getattr(wl, "loss_kind", "mse"))


def _ptr(t: Optional[torch.Tensor], dtype, what: str) -> Optional[int]:
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a tensor on the GPU" % what)
    if t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (what, dtype, t.dtype))
    if not t.is_contiguous():
        raise TypeError("%s must be contiguous" % what)
    return t.data_ptr()


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


class Params:
    """Device-resident parameters.  Keeps the tensors alive next to the ``ab_params`` struct.

    ``W``/``b`` are lists in the ABI's layer order (tensor-encoder layers first, then hidden layers,
    then the output layer).  With ``trainable=True`` fp32 masters and zeroed Adam moments are added.
    """

    def __init__(self, W: Sequence, b: Sequence, dtype: str, device="cuda:0", trainable: bool = False):
        cdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.dtype = dtype
        as_t = lambda a: a if isinstance(a, torch.Tensor) else torch.from_numpy(a)
        self.W = [as_t(w).to(device=device, dtype=torch.float32).to(cdt).contiguous() for w in W]
        self.b = [as_t(x).to(device=device, dtype=torch.float32).contiguous() for x in b]
        self.c = ab_params()
        for k, (w, x) in enumerate(zip(self.W, self.b)):
            self.c.W[k] = w.data_ptr()
            self.c.b[k] = x.data_ptr()
        self.W_master = self.mW = self.vW = self.mb = self.vb = None
        self.step = None
        if trainable:
            self.W_master = [as_t(w).to(device=device, dtype=torch.float32).contiguous().clone() for w in W]
            z = lambda xs: [torch.zeros_like(x) for x in xs]
            self.mW, self.vW, self.mb, self.vb = z(self.W_master), z(self.W_master), z(self.b), z(self.b)
            self.step = torch.zeros(1, dtype=torch.int64, device=device)
            for k in range(len(self.W)):
                self.c.W_master[k] = self.W_master[k].data_ptr()
                self.c.adam_mW[k] = self.mW[k].data_ptr()
                self.c.adam_vW[k] = self.vW[k].data_ptr()
                self.c.adam_mb[k] = self.mb[k].data_ptr()
                self.c.adam_vb[k] = self.vb[k].data_ptr()
            self.c.step = self.step.data_ptr()

    @staticmethod
    def from_workload(wl, device="cuda:0", trainable=False) -> "Params":
        W = list(getattr(wl, "te_W", None) or []) + list(wl.W)
        b = list(getattr(wl, "te_b", None) or []) + list(wl.b)
        return Params(W, b, wl.dtype, device, trainable)


# ---------------------------------------------------------------------------------------------
# the entry points
# ---------------------------------------------------------------------------------------------
def ab_workspace_bytes(desc: ab_model_desc, S: int = 0, C_: int = 0, B: int = 0) -> int:
    return int(load().ab_workspace_bytes(C.byref(desc), int(S), int(C_), int(B)))


def alloc_workspace(desc: ab_model_desc, S: int = 0, C_: int = 0, B: int = 0, device="cuda:0") -> torch.Tensor:
    n = ab_workspace_bytes(desc, S, C_, B)
    if n == 0:
        raise AutoByteError(-6, "ab_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def ab_score_candidates(desc: ab_model_desc, params: Params, dyn: torch.Tensor, scalars: torch.Tensor,
                        partition_bytes: torch.Tensor, credit_mult: torch.Tensor,
                        scores: Optional[torch.Tensor] = None, best_idx: Optional[torch.Tensor] = None,
                        best_score: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                        stream=None, check: bool = True, layers_of: Optional[torch.Tensor] = None,
                        static_scratch: bool = False, v_best: Optional[torch.Tensor] = None) -> int:
    """Enqueue scoring of every (scenario, candidate); outputs are written into the given tensors.
    ``v_best`` [S, n_outputs] (needs ``best_idx``): the predicted speed vector of the chosen candidate.
    ``layers_of`` (int32 [S], encoder models only): how many of the L padded layers each scenario really has.
    ``partition_bytes`` [P] and ``credit_mult`` [Q] are shared by all scenarios; given as [S, P] and [S, Q]
    every scenario brings its own grid."""
    lib = load()
    S = int(dyn.shape[0])
    if layers_of is not None and layers_of.numel() != S:
        raise ValueError("layers_of must have one entry per scenario")
    st = ab_stats(_ptr(dyn, torch.float32, "dyn"), _ptr(scalars, torch.float32, "scalars"), S,
                  _ptr(layers_of, torch.int32, "layers_of"))
    per_scenario = partition_bytes.dim() == 2
    if per_scenario and (credit_mult.dim() != 2 or partition_bytes.shape[0] != S or credit_mult.shape[0] != S):
        raise ValueError("per-scenario grids must be [S, P] and [S, Q]")
    P, Q = int(partition_bytes.shape[-1]), int(credit_mult.shape[-1])
    gr = ab_grid(_ptr(partition_bytes, torch.float32, "partition_bytes"), P,
                 _ptr(credit_mult, torch.float32, "credit_mult"), Q, 1 if per_scenario else 0)
    if dyn.numel() != S * desc.n_layers * desc.n_stats or scalars.numel() != S * desc.n_scalars:
        raise ValueError("dyn / scalars do not match the description")
    for t, n, what in ((scores, S * P * Q, "scores"), (best_idx, S, "best_idx"), (best_score, S, "best_score")):
        if t is not None and t.numel() != n:
            raise ValueError("%s has %d elements, expected %d" % (what, t.numel(), n))
    n_out = max(1, int(desc.n_outputs))
    if v_best is not None and v_best.numel() != S * n_out:
        raise ValueError("v_best has %d elements, expected %d" % (v_best.numel(), S * n_out))
    if static_scratch:
        if workspace is not None or v_best is not None:
            raise ValueError("the static-scratch form takes neither a workspace nor v_best")
        rc = lib.ab_score_candidates_static(C.byref(desc), C.byref(params.c), C.byref(st), C.byref(gr),
                                            _ptr(scores, torch.float32, "scores"),
                                            _ptr(best_idx, torch.int32, "best_idx"),
                                            _ptr(best_score, torch.float32, "best_score"), _stream_handle(stream))
        if check and rc != 0:
            raise AutoByteError(rc, "ab_score_candidates_static")
        return rc
    ws_ptr = _ptr(workspace, torch.uint8, "workspace")
    if v_best is not None:
        rc = lib.ab_score_candidates_v(C.byref(desc), C.byref(params.c), C.byref(st), C.byref(gr),
                                       _ptr(scores, torch.float32, "scores"), _ptr(best_idx, torch.int32, "best_idx"),
                                       _ptr(best_score, torch.float32, "best_score"),
                                       _ptr(v_best, torch.float32, "v_best"), ws_ptr,
                                       0 if workspace is None else workspace.numel(), _stream_handle(stream))
        if check and rc != 0:
            raise AutoByteError(rc, "ab_score_candidates_v")
        return rc
    rc = lib.ab_score_candidates(C.byref(desc), C.byref(params.c), C.byref(st), C.byref(gr),
                                 _ptr(scores, torch.float32, "scores"), _ptr(best_idx, torch.int32, "best_idx"),
                                 _ptr(best_score, torch.float32, "best_score"), ws_ptr,
                                 0 if workspace is None else workspace.numel(), _stream_handle(stream))
    if check and rc != 0:
        raise AutoByteError(rc, "ab_score_candidates")
    return rc


def ab_score_candidates_static(desc: ab_model_desc, params: Params, dyn: torch.Tensor, scalars: torch.Tensor,
                               partition_bytes: torch.Tensor, credit_mult: torch.Tensor,
                               scores: Optional[torch.Tensor] = None, best_idx: Optional[torch.Tensor] = None,
                               best_score: Optional[torch.Tensor] = None, stream=None, check: bool = True,
                               layers_of: Optional[torch.Tensor] = None) -> int:
    """``ab_score_candidates`` on the library's fixed scratch array: no workspace, nothing allocated."""
    return ab_score_candidates(desc, params, dyn, scalars, partition_bytes, credit_mult, scores, best_idx,
                               best_score, None, stream, check, layers_of, static_scratch=True)


def ab_static_scratch_bytes() -> int:
    return int(load().ab_static_scratch_bytes())


def ab_select_best(scores: torch.Tensor, best_idx: torch.Tensor, best_score: Optional[torch.Tensor] = None,
                   C_: Optional[int] = None, row_stride: Optional[int] = None, stream=None,
                   check: bool = True) -> int:
    """Per-row argmax of ``scores`` [S, row_stride] over the first ``C_`` columns."""
    lib = load()
    if scores.dim() != 2:
        raise ValueError("scores must be 2-D")
    S = int(scores.shape[0])
    row_stride = int(scores.shape[1]) if row_stride is None else int(row_stride)
    C_ = row_stride if C_ is None else int(C_)
    if best_idx.numel() != S or (best_score is not None and best_score.numel() != S):
        raise ValueError("best_idx / best_score must have one element per row")
    rc = lib.ab_select_best(_ptr(scores, torch.float32, "scores"), S, C_, row_stride,
                            _ptr(best_idx, torch.int32, "best_idx"),
                            _ptr(best_score, torch.float32, "best_score"), _stream_handle(stream))
    if check and rc != 0:
        raise AutoByteError(rc, "ab_select_best")
    return rc


def ab_trigger(scores: torch.Tensor, current_idx: torch.Tensor, best_idx: torch.Tensor,
               reconfigure: torch.Tensor, observed: Optional[torch.Tensor] = None,
               gain: Optional[torch.Tensor] = None, adapt: Optional[torch.Tensor] = None,
               gain_threshold: float = 0.05, error_threshold: float = 0.10, C_: Optional[int] = None,
               row_stride: Optional[int] = None, stream=None, check: bool = True) -> int:
    """Choice plus the Optimization Trigger's two threshold tests on ``scores`` [S, row_stride]."""
    lib = load()
    if scores.dim() != 2:
        raise ValueError("scores must be 2-D")
    S = int(scores.shape[0])
    row_stride = int(scores.shape[1]) if row_stride is None else int(row_stride)
    C_ = row_stride if C_ is None else int(C_)
    for t, what in ((current_idx, "current_idx"), (best_idx, "best_idx"), (reconfigure, "reconfigure"),
                    (observed, "observed"), (gain, "gain"), (adapt, "adapt")):
        if t is not None and t.numel() != S:
            raise ValueError("%s must have one element per row" % what)
    rc = lib.ab_trigger(_ptr(scores, torch.float32, "scores"), S, C_, row_stride,
                        _ptr(current_idx, torch.int32, "current_idx"), _ptr(observed, torch.float32, "observed"),
                        gain_threshold, error_threshold, _ptr(best_idx, torch.int32, "best_idx"),
                        _ptr(gain, torch.float32, "gain"), _ptr(reconfigure, torch.uint8, "reconfigure"),
                        _ptr(adapt, torch.uint8, "adapt"), _stream_handle(stream))
    if check and rc != 0:
        raise AutoByteError(rc, "ab_trigger")
    return rc


def ab_online_update(desc: ab_model_desc, params: Params, x_raw: torch.Tensor, target: torch.Tensor,
                     lr: float = 1e-3, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                     loss_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                     stream=None, check: bool = True) -> int:
    """Enqueue one forward + backward + Adam step on the rows of ``x_raw`` [B, F]."""
    lib = load()
    B = int(x_raw.shape[0])
    F = desc.n_layers * desc.n_stats + desc.n_scalars + 2
    if x_raw.numel() != B * F or target.numel() != B * max(1, int(desc.n_outputs)):
        raise ValueError("x_raw must be [B, %d] and target [B, n_outputs]" % F)
    if params.step is None:
        raise ValueError("params were not created with trainable=True")
    rc = lib.ab_online_update(C.byref(desc), C.byref(params.c), _ptr(x_raw, torch.float32, "x_raw"),
                              _ptr(target, torch.float32, "target"), B, lr, beta1, beta2, eps,
                              _ptr(loss_out, torch.float32, "loss_out"),
                              _ptr(workspace, torch.uint8, "workspace"),
                              0 if workspace is None else workspace.numel(), _stream_handle(stream))
    if check and rc != 0:
        raise AutoByteError(rc, "ab_online_update")
    return rc


def ab_online_update_tail(desc: ab_model_desc, params: Params, x_raw: torch.Tensor, target: torch.Tensor,
                          first_trainable: int, lr: float = 1e-3, beta1: float = 0.9, beta2: float = 0.999,
                          eps: float = 1e-8, loss_out: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None, stream=None, check: bool = True) -> int:
    """The online step with scorer layers below ``first_trainable`` frozen."""
    lib = load()
    B = int(x_raw.shape[0])
    F = desc.n_layers * desc.n_stats + desc.n_scalars + 2
    if x_raw.numel() != B * F or target.numel() != B * max(1, int(desc.n_outputs)):
        raise ValueError("x_raw must be [B, %d] and target [B, n_outputs]" % F)
    if params.step is None:
        raise ValueError("params were not created with trainable=True")
    rc = lib.ab_online_update_tail(C.byref(desc), C.byref(params.c), _ptr(x_raw, torch.float32, "x_raw"),
                                   _ptr(target, torch.float32, "target"), B, int(first_trainable),
                                   lr, beta1, beta2, eps, _ptr(loss_out, torch.float32, "loss_out"),
                                   _ptr(workspace, torch.uint8, "workspace"),
                                   0 if workspace is None else workspace.numel(), _stream_handle(stream))
    if check and rc != 0:
        raise AutoByteError(rc, "ab_online_update_tail")
    return rc


def ab_replay_mix(x_new: Optional[torch.Tensor], target_new: Optional[torch.Tensor], x_old: Optional[torch.Tensor],
                  target_old: Optional[torch.Tensor], pick: torch.Tensor, x_out: torch.Tensor,
                  target_out: torch.Tensor, stream=None, check: bool = True) -> int:
    """Gather a minibatch from a pool of new rows (pick >= 0) and a pool of old rows (pick < 0: row -pick-1)."""
    lib = load()
    B, F = int(x_out.shape[0]), int(x_out.shape[1])
    n_new = 0 if x_new is None else int(x_new.shape[0])
    n_old = 0 if x_old is None else int(x_old.shape[0])
    for t_ in (x_new, x_old):
        if t_ is not None and int(t_.shape[1]) != F:
            raise ValueError("pools and output must have the same row width")
    if pick.numel() != B or target_out.numel() % B != 0:
        raise ValueError("pick must have one entry and target_out n_outputs entries per output row")
    n_out = target_out.numel() // B
    for t_, n_ in ((target_new, n_new), (target_old, n_old)):
        if t_ is not None and t_.numel() != n_ * n_out:
            raise ValueError("pool targets must have %d entries per row" % n_out)
    rc = lib.ab_replay_mix(_ptr(x_new, torch.float32, "x_new"), _ptr(target_new, torch.float32, "target_new"), n_new,
                           _ptr(x_old, torch.float32, "x_old"), _ptr(target_old, torch.float32, "target_old"), n_old,
                           _ptr(pick, torch.int32, "pick"), B, F, n_out, _ptr(x_out, torch.float32, "x_out"),
                           _ptr(target_out, torch.float32, "target_out"), _stream_handle(stream))
    if check and rc != 0:
        raise AutoByteError(rc, "ab_replay_mix")
    return rc
