"""Seeded synthetic inputs shaped like the AutoByte workloads.

This module only *draws data*: raw runtime statistics, candidate grids, network weights, training
targets.  It contains none of the meta-network's arithmetic (no feature transform, no layer, no
argmax, no optimiser), so that the CPU oracle and the GPU library can both be fed from it without
sharing any of the method.  The feature-transform constants it hands out are plain numbers that
describe the distributions drawn here (location / spread of each raw quantity); in a deployment
they would be fitted offline together with the weights.

Shapes and ranges follow the paper's data collection (arXiv 2112.13509, Section 3.2 "Dataset
collection": partition size and credit multiple grids, bandwidth range, three CNN models) and
Table 1 (worker count, model / architecture type, per-layer computation time, bandwidth), widened
to batched "many scenarios x many candidates" service sizes.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

ENC_LINEAR, ENC_LOG = 0, 1
KIB, MIB = 1024.0, 1024.0 * 1024.0
BASE_SEED = 211213509

Enc = Tuple[int, float, float]


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    out = r.view(np.float32).copy()
    nan = np.isnan(a)
    out[nan] = np.nan
    return out.reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already bfloat16-representable float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def log_spaced(lo: float, hi: float, n: int) -> np.ndarray:
    """v_i = lo * (hi/lo)^(i/(n-1)) in float64, cast to float32."""
    if n == 1:
        return np.asarray([lo], dtype=np.float32)
    i = np.arange(n, dtype=np.float64)
    return (lo * (hi / lo) ** (i / (n - 1))).astype(np.float32)


def _log_uniform_enc(lo: float, hi: float) -> Enc:
    """Constants that standardise ln(x) for x log-uniform on [lo, hi] (unit variance, zero mean)."""
    if hi <= lo:
        return (ENC_LOG, math.log(lo), 1.0)
    return (ENC_LOG, 0.5 * (math.log(lo) + math.log(hi)), math.sqrt(12.0) / (math.log(hi) - math.log(lo)))


@dataclass
class Workload:
    """One scoring problem: model description + weights + raw inputs (all NumPy, float32 values)."""
    name: str
    dtype: str                      # "f32" or "bf16": the arithmetic type the GPU path computes in
    L: int
    K: int
    stat_enc: List[Enc]
    scal_enc: List[Enc]
    part_enc: Enc
    cred_enc: Enc
    hidden: List[int]
    W: List[np.ndarray]             # [out, in] float32 (bf16-representable when dtype == "bf16")
    b: List[np.ndarray]             # float32
    te_hidden: Optional[List[int]]  # tensor encoder widths or None
    te_W: Optional[List[np.ndarray]]
    te_b: Optional[List[np.ndarray]]
    dyn: np.ndarray                 # [S, L, K] float32 raw statistics
    scal: np.ndarray                # [S, Ns] float32 raw scalars
    part: np.ndarray                # [P] float32 partition sizes in bytes
    cred: np.ndarray                # [Q] float32 credit multiples
    seed: int = 0
    te_kind: str = "mlp"            # "mlp": per-layer MLP + mean; "lstm": embedding + two-layer LSTM over the layers

    @property
    def S(self) -> int:
        return self.dyn.shape[0]

    @property
    def C(self) -> int:
        return self.part.shape[0] * self.cred.shape[0]

    @property
    def Ns(self) -> int:
        return len(self.scal_enc)

    @property
    def F(self) -> int:
        return (self.te_hidden[1] if self.te_hidden else self.L * self.K) + self.Ns + 2   # (te_hidden = [E, H] for "lstm")

    def subset(self, idx) -> "Workload":
        """Same model and grid, scenarios restricted to ``idx``."""
        idx = np.asarray(idx)
        return Workload(self.name, self.dtype, self.L, self.K, self.stat_enc, self.scal_enc,
                        self.part_enc, self.cred_enc, self.hidden, self.W, self.b, self.te_hidden,
                        self.te_W, self.te_b, np.ascontiguousarray(self.dyn[idx]),
                        np.ascontiguousarray(self.scal[idx]), self.part, self.cred, self.seed, self.te_kind)


# --------------------------------------------------------------------------------------------
# raw statistics
# --------------------------------------------------------------------------------------------
TIME_MU, TIME_SIGMA = math.log(2.0), 0.5          # lognormal compute time, median 2 ms
WORKER_CHOICES = np.asarray([2.0, 4.0, 8.0, 16.0])
BW_LO, BW_HI = 1.0, 100.0                          # Gbps


def _time_enc() -> Enc:
    return (ENC_LOG, TIME_MU, 1.0 / TIME_SIGMA)


def _scalar_encs(n_onehot_groups: int) -> List[Enc]:
    lw = np.log(WORKER_CHOICES)
    encs: List[Enc] = [(ENC_LOG, float(lw.mean()), float(1.0 / lw.std())),
                       (ENC_LINEAR, 0.5 * (BW_LO + BW_HI), math.sqrt(12.0) / (BW_HI - BW_LO))]
    encs += [(ENC_LINEAR, 0.0, 1.0)] * (2 * n_onehot_groups)
    return encs


def _draw_scalars(rng: np.random.Generator, S: int, n_onehot_groups: int):
    """workers, bandwidth, then 2-way one-hots (model type[, architecture type]).
    Returns raw values and the standardised latents they were made from."""
    wi = rng.integers(0, 4, size=S)
    workers = WORKER_CHOICES[wi]
    ub = rng.random(S)
    bw = BW_LO + (BW_HI - BW_LO) * ub
    cols = [workers, bw]
    lat = [(wi - 1.5) / math.sqrt(1.25), (ub - 0.5) * math.sqrt(12.0)]
    for _ in range(n_onehot_groups):
        t = rng.integers(0, 2, size=S)
        cols += [(t == 0).astype(np.float64), (t == 1).astype(np.float64)]
        lat += [(t == 0).astype(np.float64), (t == 1).astype(np.float64)]
    return np.stack(cols, axis=1).astype(np.float32), np.stack(lat, axis=1)


def _draw_layer_stats(rng: np.random.Generator, S: int, L: int, bytes_lo: float, bytes_hi: float):
    """[S, L, 3]: forward ms, backward ms, tensor bytes; plus standardised latents."""
    zf = rng.standard_normal((S, L))
    zb = rng.standard_normal((S, L))
    ub = rng.random((S, L))
    fwd = np.exp(TIME_MU + TIME_SIGMA * zf)
    bwd = np.exp(TIME_MU + TIME_SIGMA * zb)
    nbytes = np.exp(math.log(bytes_lo) + (math.log(bytes_hi) - math.log(bytes_lo)) * ub)
    dyn = np.stack([fwd, bwd, nbytes], axis=2).astype(np.float32)
    lat = np.stack([zf, zb, (ub - 0.5) * math.sqrt(12.0)], axis=2)
    return dyn, lat


def _draw_transformer_stats(rng: np.random.Generator, S: int, n_blocks=24, per_block=16, extra=16,
                            bytes_lo=1.0 * KIB, bytes_hi=256.0 * MIB):
    """[S, L, 4] with L = n_blocks*per_block + extra: forward ms, backward ms, bytes, position.
    Tensor sizes repeat from block to block (one draw of ``per_block`` sizes per scenario);
    the trailing ``extra`` tensors (embeddings and the like) are drawn independently.
    Compute times are i.i.d. lognormal per tensor."""
    L = n_blocks * per_block + extra
    span = math.log(bytes_hi) - math.log(bytes_lo)
    ub_block = rng.random((S, per_block))
    ub_extra = rng.random((S, extra))
    ub = np.concatenate([np.tile(ub_block, (1, n_blocks)), ub_extra], axis=1)
    nbytes = np.exp(math.log(bytes_lo) + span * ub)
    fwd = np.exp(TIME_MU + TIME_SIGMA * rng.standard_normal((S, L)))
    bwd = np.exp(TIME_MU + TIME_SIGMA * rng.standard_normal((S, L)))
    pos = np.broadcast_to(np.arange(L, dtype=np.float64) / max(L - 1, 1), (S, L))
    return np.stack([fwd, bwd, nbytes, pos], axis=2).astype(np.float32)


def _draw_dense(rng: np.random.Generator, n_out: int, n_in: int, dtype: str):
    """W ~ N(0, 1/fan_in) (variance), b ~ N(0, 0.1^2)."""
    W = (rng.standard_normal((n_out, n_in)) / math.sqrt(n_in)).astype(np.float32)
    b = (0.1 * rng.standard_normal(n_out)).astype(np.float32)
    if dtype == "bf16":
        W = bf16_round(W)
    return W, b


def _draw_mlp(rng, widths: List[int], dtype: str):
    Ws, bs = [], []
    for k in range(len(widths) - 1):
        W, b = _draw_dense(rng, widths[k + 1], widths[k], dtype)
        Ws.append(W)
        bs.append(b)
    return Ws, bs


def make_scoring(name: str, S: int, L: int, hidden: List[int], P: int, Q: int,
                 part_lo: float, part_hi: float, cred_lo: float, cred_hi: float,
                 cred_integer: bool, dtype: str, seed: int,
                 bytes_lo: float = 4.0 * KIB, bytes_hi: float = 400.0 * MIB) -> Workload:
    """Flat-feature scoring problem (L layers x 3 statistics + workers, bandwidth, model one-hot)."""
    rng = np.random.default_rng(seed)
    Ws, bs = _draw_mlp(rng, [L * 3 + 4 + 2] + list(hidden) + [1], dtype)
    dyn, _ = _draw_layer_stats(rng, S, L, bytes_lo, bytes_hi)
    scal, _ = _draw_scalars(rng, S, 1)
    part = log_spaced(part_lo, part_hi, P)
    cred = (np.linspace(cred_lo, cred_hi, Q).astype(np.float32) if cred_integer
            else log_spaced(cred_lo, cred_hi, Q))
    stat_enc = [_time_enc(), _time_enc(), _log_uniform_enc(bytes_lo, bytes_hi)]
    return Workload(name, dtype, L, 3, stat_enc, _scalar_encs(1),
                    _log_uniform_enc(part_lo, part_hi), _log_uniform_enc(cred_lo, cred_hi),
                    list(hidden), Ws, bs, None, None, None, dyn, scal, part, cred, seed)


def make_integer_scoring(name: str, S: int, L: int, hidden: List[int], P: int, Q: int, dtype: str, seed: int,
                         nonzeros: int = 8) -> Workload:
    """Flat-feature scoring problem in small integers, for tests that want arithmetic without rounding: raw
    statistics, scalars and grid values are integers in 0..2 under the identity transform, every weight row
    holds ``nonzeros`` entries of +-1 (half of each sign, at seeded positions; the rest zero), biases are in
    {-1, 0, 1}.  With few non-zeros per row the activations stay small integers, which bf16 and fp32 both
    hold exactly (the caller checks that on its reference), so every summation order gives the same result."""
    rng = np.random.default_rng(seed)
    widths = [L * 3 + 4 + 2] + list(hidden) + [1]
    Ws, bs = [], []
    for k in range(len(widths) - 1):
        n_out, n_in = widths[k + 1], widths[k]
        nz = min(nonzeros, n_in // 2 * 2)
        W = np.zeros((n_out, n_in), dtype=np.float32)
        for o in range(n_out):
            cols = rng.choice(n_in, size=nz, replace=False)
            W[o, cols[:nz // 2]] = 1.0
            W[o, cols[nz // 2:]] = -1.0
        Ws.append(W)
        bs.append(rng.integers(-1, 2, n_out).astype(np.float32))
    dyn = rng.integers(0, 3, (S, L, 3)).astype(np.float32)
    scal = rng.integers(0, 3, (S, 4)).astype(np.float32)
    part = rng.integers(0, 3, P).astype(np.float32)
    cred = rng.integers(0, 3, Q).astype(np.float32)
    lin = (ENC_LINEAR, 0.0, 1.0)
    return Workload(name, dtype, L, 3, [lin] * 3, [lin] * 4, lin, lin, list(hidden), Ws, bs, None, None, None,
                    dyn, scal, part, cred, seed)


def make_per_worker(name: str, S: int, L: int, n_workers: int, hidden: List[int], P: int, Q: int,
                    dtype: str, seed: int) -> Workload:
    """Scoring problem with the input record of Table 1: per layer the backward time on each of the
    ``n_workers`` workers (T is l x n: a layer's base time ~ lognormal(ln 2 ms, 0.5), times a per-worker speed
    factor ~ lognormal(0, 0.1), times a per-sample jitter ~ lognormal(0, 0.05)); scalars n, l, a 2-way model-type
    and a 2-way architecture-type vector, then the download and the upload speed of every worker (B_d, B_u:
    U(1, 100) Gbps each); the output layer predicts one speed per worker."""
    rng = np.random.default_rng(seed)
    Ns = 2 + 4 + 2 * n_workers
    Ws, bs = _draw_mlp(rng, [L * n_workers + Ns + 2] + list(hidden) + [n_workers], dtype)
    base = np.exp(TIME_MU + TIME_SIGMA * rng.standard_normal((S, L, 1)))
    dyn = (base * np.exp(0.1 * rng.standard_normal((S, 1, n_workers)))
           * np.exp(0.05 * rng.standard_normal((S, L, n_workers)))).astype(np.float32)
    t1, t2 = rng.integers(0, 2, size=S), rng.integers(0, 2, size=S)
    cols = [np.full(S, float(n_workers)), np.full(S, float(L)), t1 == 0, t1 == 1, t2 == 0, t2 == 1]
    bw = BW_LO + (BW_HI - BW_LO) * rng.random((S, 2 * n_workers))
    scal = np.concatenate([np.stack(cols, axis=1).astype(np.float64), bw], axis=1).astype(np.float32)
    bw_enc = (ENC_LINEAR, 0.5 * (BW_LO + BW_HI), math.sqrt(12.0) / (BW_HI - BW_LO))
    scal_enc = [(ENC_LOG, math.log(8.0), 1.0), (ENC_LINEAR, 64.0, 1.0 / 64.0)] + [(ENC_LINEAR, 0.0, 1.0)] * 4 \
        + [bw_enc] * (2 * n_workers)
    part_lo, part_hi, cred_lo, cred_hi = 16.0 * KIB, 64.0 * MIB, 1.0, 64.0
    return Workload(name, dtype, L, n_workers, [_time_enc()] * n_workers, scal_enc,
                    _log_uniform_enc(part_lo, part_hi), _log_uniform_enc(cred_lo, cred_hi),
                    list(hidden), Ws, bs, None, None, None, dyn, scal,
                    log_spaced(part_lo, part_hi, P), log_spaced(cred_lo, cred_hi, Q), seed)


def make_tensor_encoder(name: str, S: int, hidden: List[int], te_hidden: List[int], P: int, Q: int,
                        dtype: str, seed: int, n_blocks=24, per_block=16, extra=16) -> Workload:
    """Per-tensor-encoder scoring problem (transformer-like tensor list, 4 statistics per tensor,
    six scalars: workers, bandwidth, model one-hot, architecture one-hot)."""
    rng = np.random.default_rng(seed)
    te_W, te_b = _draw_mlp(rng, [4] + list(te_hidden), dtype)
    Ws, bs = _draw_mlp(rng, [te_hidden[1] + 6 + 2] + list(hidden) + [1], dtype)
    dyn = _draw_transformer_stats(rng, S, n_blocks, per_block, extra)
    scal, _ = _draw_scalars(rng, S, 2)
    part_lo, part_hi, cred_lo, cred_hi = 16.0 * KIB, 64.0 * MIB, 1.0, 64.0
    stat_enc = [_time_enc(), _time_enc(), _log_uniform_enc(1.0 * KIB, 256.0 * MIB),
                (ENC_LINEAR, 0.5, math.sqrt(12.0))]
    return Workload(name, dtype, dyn.shape[1], 4, stat_enc, _scalar_encs(2),
                    _log_uniform_enc(part_lo, part_hi), _log_uniform_enc(cred_lo, cred_hi),
                    list(hidden), Ws, bs, list(te_hidden), te_W, te_b, dyn, scal,
                    log_spaced(part_lo, part_hi, P), log_spaced(cred_lo, cred_hi, Q), seed)


def make_integer_tensor_encoder(name: str, S: int, L: int, hidden: List[int], P: int, Q: int, dtype: str,
                                seed: int, kinds: int = 2, alternate: bool = False) -> Workload:
    """The per-tensor-encoder problem in small integers (see ``make_integer_scoring``): 4 integer statistics per
    tensor under the identity transform, encoder 4 -> 128 -> 128 and scorer with a few +-1 weights per row.  A
    scenario's L tensors (L a multiple of ``kinds``) are ``kinds`` distinct ones, each L / kinds times, in a seeded
    order, so that the mean over the tensors is a multiple of 1 / kinds: with kinds = 2 and L a power of two the
    pooled block keeps one fractional bit and stays exactly representable.  With ``alternate`` the kinds take turns
    (0, 1, 0, 1, ...), so that every prefix of a length that is a multiple of ``kinds`` is balanced as well."""
    assert L % kinds == 0
    rng = np.random.default_rng(seed)

    def sparse(n_out, n_in, nz):
        W = np.zeros((n_out, n_in), dtype=np.float32)
        nz = min(nz, n_in // 2 * 2)
        for o in range(n_out):
            cols = rng.choice(n_in, size=nz, replace=False)
            W[o, cols[:nz // 2]] = 1.0
            W[o, cols[nz // 2:]] = -1.0
        return W, rng.integers(-1, 2, n_out).astype(np.float32)

    Wa, ba = sparse(128, 4, 2)
    Wb, bb = sparse(128, 128, 4)
    widths = [128 + 6 + 2] + list(hidden) + [1]
    Ws, bs = [], []
    for k in range(len(widths) - 1):
        W, b = sparse(widths[k + 1], widths[k], 8)
        Ws.append(W)
        bs.append(b)
    proto = rng.integers(0, 3, (S, kinds, 4)).astype(np.float32)
    order = np.stack([rng.permutation(np.repeat(np.arange(kinds), L // kinds)) for _ in range(S)])
    if alternate:
        order = np.tile(np.arange(L) % kinds, (S, 1))
    dyn = np.take_along_axis(proto, order[:, :, None].repeat(4, axis=2), axis=1)
    scal = rng.integers(0, 3, (S, 6)).astype(np.float32)
    lin = (ENC_LINEAR, 0.0, 1.0)
    return Workload(name, dtype, L, 4, [lin] * 4, [lin] * 6, lin, lin, list(hidden), Ws, bs, [128, 128],
                    [Wa, Wb], [ba, bb], np.ascontiguousarray(dyn), scal,
                    rng.integers(0, 3, P).astype(np.float32), rng.integers(0, 3, Q).astype(np.float32), seed)


def make_lstm_encoder(name: str, S: int, hidden: List[int], P: int, Q: int, dtype: str, seed: int,
                      n_blocks=24, per_block=16, extra=16, E: int = 32, H: int = 64) -> Workload:
    """The tensor-encoder problem with the temporal encoder in front: per-tensor statistics embedded into E
    values, two LSTM layers of H units over the tensor sequence (te_W = [[E,4], [4H,E+H], [4H,2H]])."""
    rng = np.random.default_rng(seed)
    W_e, b_e = _draw_dense(rng, E, 4, dtype)
    W_1, b_1 = _draw_dense(rng, 4 * H, E + H, dtype)
    W_2, b_2 = _draw_dense(rng, 4 * H, 2 * H, dtype)
    Ws, bs = _draw_mlp(rng, [H + 6 + 2] + list(hidden) + [1], dtype)
    dyn = _draw_transformer_stats(rng, S, n_blocks, per_block, extra)
    scal, _ = _draw_scalars(rng, S, 2)
    part_lo, part_hi, cred_lo, cred_hi = 16.0 * KIB, 64.0 * MIB, 1.0, 64.0
    stat_enc = [_time_enc(), _time_enc(), _log_uniform_enc(1.0 * KIB, 256.0 * MIB),
                (ENC_LINEAR, 0.5, math.sqrt(12.0))]
    return Workload(name, dtype, dyn.shape[1], 4, stat_enc, _scalar_encs(2),
                    _log_uniform_enc(part_lo, part_hi), _log_uniform_enc(cred_lo, cred_hi),
                    list(hidden), Ws, bs, [E, H], [W_e, W_1, W_2], [b_e, b_1, b_2], dyn, scal,
                    log_spaced(part_lo, part_hi, P), log_spaced(cred_lo, cred_hi, Q), seed, "lstm")


def make_config(cfg: int, S: Optional[int] = None, seed: Optional[int] = None) -> Workload:
    """The four scoring configurations (1, 2, 3, 5).  ``S`` overrides the scenario count (the
    distributions, model and grid stay those of the configuration)."""
    seed = BASE_SEED + cfg if seed is None else seed
    if cfg == 1:
        return make_scoring("cfg1-tiny-f32", S or 1, 16, [64, 64], 8, 8, 64 * KIB, 64 * MIB,
                            1.0, 8.0, True, "f32", seed)
    if cfg == 2:
        return make_scoring("cfg2-batch-f32", S or 1024, 128, [256, 256], 64, 64, 16 * KIB, 64 * MIB,
                            1.0, 64.0, False, "f32", seed)
    if cfg == 3:
        return make_scoring("cfg3-mfma-bf16", S or 65536, 128, [1024] * 4, 16, 16, 16 * KIB, 64 * MIB,
                            1.0, 64.0, False, "bf16", seed)
    if cfg == 5:
        return make_tensor_encoder("cfg5-tensor-encoder-bf16", S or 8192, [512, 512], [128, 128],
                                   32, 32, "bf16", seed)
    if cfg == 6:     # not one of the five baseline configurations: configuration 5's shape with the paper's LSTM encoder
        return make_lstm_encoder("lstm-encoder-bf16", S or 8192, [512, 512], 32, 32, "bf16", seed)
    raise ValueError("scoring configurations are 1, 2, 3, 5 and 6 (4 is the update workload)")


def sample_scenarios(S: int, n_first: int, n_last: int, n_mid: int, edge: int, seed: int) -> np.ndarray:
    """Scenario indices for a reference sample of a full-size run: the first ``n_first``, the last ``n_last``
    and ``n_mid`` in between, of which as many as fit sit on both sides of a multiple of ``edge`` (the number
    of scenarios one chunk of the launch sequence holds, so the last tile of one chunk and the first of the
    next are both looked at); the rest are seeded random draws.  Sorted, without repeats."""
    rng = np.random.default_rng(seed)
    borders = np.arange(edge, S, edge, dtype=np.int64)
    mid = np.concatenate([borders - 1, borders])
    if mid.size > n_mid:
        mid = rng.choice(mid, n_mid, replace=False)
    lo, hi = min(n_first, S), max(min(n_first, S) + 1, S - n_last)
    extra = rng.integers(lo, hi, max(0, n_mid - mid.size)) if hi > lo else np.zeros(0, dtype=np.int64)
    rows = np.concatenate([np.arange(min(n_first, S)), np.arange(max(0, S - n_last), S), mid, extra])
    return np.unique(rows[(rows >= 0) & (rows < S)].astype(np.int64))


# --------------------------------------------------------------------------------------------
# online-adaptation workload
# --------------------------------------------------------------------------------------------
@dataclass
class UpdateWorkload:
    """Sample pool + minibatch order for the online-adaptation update."""
    name: str
    dtype: str
    L: int
    K: int
    stat_enc: List[Enc]
    scal_enc: List[Enc]
    part_enc: Enc
    cred_enc: Enc
    hidden: List[int]
    W: List[np.ndarray]        # initial master weights, float32
    b: List[np.ndarray]
    x_raw: np.ndarray          # [N, F] float32: statistics, scalars, partition bytes, credit multiple
    target: np.ndarray         # [N] float32 observed speed-up, or [N, n_workers] (one observation per worker)
    batch: int
    seed: int
    noise_var: float
    loss_kind: str = "mse"     # "mse", or "l2norm": Euclidean norm of the per-worker error vector (Eq. 2)

    @property
    def F(self) -> int:
        return self.x_raw.shape[1]

    def batch_indices(self, step: int) -> np.ndarray:
        """Row indices of minibatch ``step`` (0-based): consecutive blocks of a per-epoch seeded
        permutation of the pool."""
        per_epoch = self.x_raw.shape[0] // self.batch
        epoch, k = divmod(step, per_epoch)
        perm = np.random.default_rng([self.seed, 7919, epoch]).permutation(self.x_raw.shape[0])
        return np.sort(perm[k * self.batch:(k + 1) * self.batch])


def make_update(name="cfg4-online-update", N=65536, batch=4096, L=128, hidden=(512, 512, 512),
                dtype="bf16", seed: Optional[int] = None, P=64, Q=64,
                noise_var=0.01, n_workers: int = 0, loss_kind: str = "mse") -> UpdateWorkload:
    """Pool of ``N`` (statistics + one configuration) rows with a synthetic observed speed-up
    ``1 + 0.3*tanh(u.z) + noise``: ``z`` are the standardised latents the raw values were drawn
    from, ``u`` ~ N(0, 1/F) is a fixed probe, noise ~ N(0, noise_var).  With ``n_workers`` > 0 the
    output layer has one unit per worker and the target one column per worker: the job's speed-up
    plus an independent N(0, noise_var) term per worker (Table 1: V has one entry per worker)."""
    seed = BASE_SEED + 4 if seed is None else seed
    rng = np.random.default_rng(seed)
    F = L * 3 + 4 + 2
    Ws, bs = _draw_mlp(rng, [F] + list(hidden) + [max(1, n_workers)], "f32")
    bytes_lo, bytes_hi = 4.0 * KIB, 400.0 * MIB
    part_lo, part_hi, cred_lo, cred_hi = 16.0 * KIB, 64.0 * MIB, 1.0, 64.0
    dyn, lat_dyn = _draw_layer_stats(rng, N, L, bytes_lo, bytes_hi)
    scal, lat_scal = _draw_scalars(rng, N, 1)
    part, cred = log_spaced(part_lo, part_hi, P), log_spaced(cred_lo, cred_hi, Q)
    pi, qi = rng.integers(0, P, size=N), rng.integers(0, Q, size=N)
    std_idx = lambda i, n: (i - 0.5 * (n - 1)) / math.sqrt((n * n - 1) / 12.0) if n > 1 else i * 0.0
    lat = np.concatenate([lat_dyn.reshape(N, L * 3), lat_scal,
                          std_idx(pi, P)[:, None], std_idx(qi, Q)[:, None]], axis=1)
    u = rng.standard_normal(F) / math.sqrt(F)
    y = 1.0 + 0.3 * np.tanh(lat @ u) + math.sqrt(noise_var) * rng.standard_normal(N)
    x_raw = np.concatenate([dyn.reshape(N, L * 3), scal, part[pi][:, None], cred[qi][:, None]],
                           axis=1).astype(np.float32)
    stat_enc = [_time_enc(), _time_enc(), _log_uniform_enc(bytes_lo, bytes_hi)]
    if n_workers > 0:
        y = y[:, None] + math.sqrt(noise_var) * rng.standard_normal((N, n_workers))
    return UpdateWorkload(name, dtype, L, 3, stat_enc, _scalar_encs(1),
                          _log_uniform_enc(part_lo, part_hi), _log_uniform_enc(cred_lo, cred_hi),
                          list(hidden), Ws, bs, x_raw, y.astype(np.float32), batch, seed, noise_var, loss_kind)


def make_integer_update(name: str, N: int, L: int, hidden, dtype: str, seed: int, nonzeros: int = 16,
                        n_workers: int = 0) -> UpdateWorkload:
    """Update rows and initial parameters in small integers (see ``make_integer_scoring``): raw values 0..2 under
    the identity transform, ``nonzeros`` entries of +-1 per weight row, biases in {-1, 0, 1}.  The target is left
    at zero for the caller to set (a test puts it a few integers away from its reference's prediction, so that
    every delta is a small multiple of 2/B)."""
    rng = np.random.default_rng(seed)
    n_out = max(1, n_workers)
    w = make_integer_scoring(name, 1, L, list(hidden), 1, 1, dtype, seed, nonzeros)
    Ws, bs = w.W, w.b
    if n_out > 1:
        Wl = np.zeros((n_out, hidden[-1]), dtype=np.float32)
        for o in range(n_out):
            cols = rng.choice(hidden[-1], size=min(nonzeros, hidden[-1] // 2 * 2), replace=False)
            Wl[o, cols[:len(cols) // 2]] = 1.0
            Wl[o, cols[len(cols) // 2:]] = -1.0
        Ws, bs = Ws[:-1] + [Wl], bs[:-1] + [rng.integers(-1, 2, n_out).astype(np.float32)]
    F = L * 3 + 4 + 2
    x_raw = rng.integers(0, 3, (N, F)).astype(np.float32)
    y = np.zeros((N, n_out) if n_workers > 0 else N, dtype=np.float32)
    return UpdateWorkload(name, dtype, L, 3, w.stat_enc, w.scal_enc, w.part_enc, w.cred_enc, list(hidden),
                          Ws, bs, x_raw, y, N, seed, 0.0, "mse")
