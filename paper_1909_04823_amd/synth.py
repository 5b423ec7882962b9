"""Seeded synthetic recommender-shaped inputs (harness only).

This module draws the *inputs* of the DES sparse hot path: CSR batches of 64-bit feature IDs
grouped in per-(sample, field) bags, labels, host-side initial weights and upstream
gradients. It holds none of the method's arithmetic: no shard function, no table hash, no row
initialiser, no operator.  The CPU oracle and the HIP library are both fed from here and
otherwise share nothing.

The workloads stand in for the datasets the paper measures on, which are not available: the
Criteo display-advertising set (26 categorical fields, Section 6 "Dataset") and an internal
set with roughly 950 feature values per sample of which 18-30 % are distinct within a batch
(Section 6 and the unique-feature table of Section 4.3).  Only their shapes are used.

Everything is a pure function of (workload index, scale, step): numpy ``PCG64`` seeded with
``SEED_BASE + index`` and one spawned child stream per step.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np

SEED_BASE = 1909_04823_00
RESERVED_KEY = np.uint64(0xFFFFFFFFFFFFFFFF)  # never emitted: the table's empty-slot marker

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_M63 = np.uint64(0x7FFFFFFFFFFFFFFF)


def scramble64(r: np.ndarray) -> np.ndarray:
    """Bijection on 64-bit integers used to turn popularity ranks into feature IDs.

    Two odd multiplications with xor-shifts in between (each step is invertible modulo 2^64),
    so distinct ranks give distinct IDs.  This is the generator's own scrambler; it is
    unrelated to the hash the table uses.
    """
    x = np.asarray(r, dtype=np.uint64).copy()
    with np.errstate(over="ignore"):
        x *= np.uint64(0xD1342543DE82EF95)
        x ^= x >> np.uint64(31)
        x *= np.uint64(0xA0761D6478BD642F)
        x ^= x >> np.uint64(29)
    return x


def scramble63(r: np.ndarray) -> np.ndarray:
    """Bijection on [0, 2^63): same construction with every step reduced modulo 2^63."""
    x = np.asarray(r, dtype=np.uint64).copy() & _M63
    with np.errstate(over="ignore"):
        x = (x * np.uint64(0xD1342543DE82EF95)) & _M63
        x ^= x >> np.uint64(31)
        x = (x * np.uint64(0xA0761D6478BD642F)) & _M63
        x ^= x >> np.uint64(29)
    return x


@dataclass(frozen=True)
class Workload:
    """One of the five measured configurations (or a shrunken copy of it for tests)."""

    index: int
    name: str
    B: int                      # samples per batch
    F: int                      # fields per sample
    D: int                      # latent dimension
    K: int                      # logical DES shards
    opt: str                    # "sgd" | "adagrad"
    lr: float
    eps: float
    bag: tuple                  # ("const", n) | ("uniform", lo, hi) | ("poisson", lam)
    key_space: int              # number of ranks the popularity law is truncated to
    preinsert: int              # ranks 1..preinsert are in the table before the first step
    capacity: int               # table capacity in rows
    zipf_a: Optional[float]     # None => uniform over key_space
    uniform_mix: float = 0.0    # fraction of entries drawn uniformly from the pre-inserted rows
    p_new: float = 0.0          # streaming: probability that an entry is a brand-new random key
    key_bits: int = 64          # 64 or 63 (IDs below 2^63)
    host_values: bool = False   # initial weights drawn on the host, N(0, init_std^2)
    init_std: float = 0.01
    pool_dense: bool = False    # keep per-shard pooled partials [K,B,F,D] (small shapes only)
    steps: int = 1

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    def rank_to_key(self, r: np.ndarray) -> np.ndarray:
        k = scramble64(r) if self.key_bits == 64 else scramble63(r)
        if np.any(k == RESERVED_KEY):
            raise ValueError("rank maps to the reserved key; change the rank range")
        return k

    def mean_bag(self) -> float:
        kind = self.bag[0]
        if kind == "const":
            return float(self.bag[1])
        if kind == "uniform":
            return 0.5 * (self.bag[1] + self.bag[2])
        lam = float(self.bag[1])
        return lam + float(np.exp(-lam))


_FULL = [
    Workload(0, "tiny_lr_fm", B=256, F=10, D=8, K=2, opt="sgd", lr=0.01, eps=0.0,
             bag=("const", 1), key_space=10_000, preinsert=10_000, capacity=16_384,
             zipf_a=None, host_values=True, pool_dense=True),
    Workload(1, "dlrm_pooled", B=4096, F=26, D=16, K=8, opt="adagrad", lr=0.05, eps=1e-8,
             bag=("uniform", 1, 20), key_space=10_000_000, preinsert=1_000_000,
             capacity=2_000_000, zipf_a=1.1, host_values=True, pool_dense=True),
    Workload(2, "deepfm", B=16384, F=100, D=32, K=16, opt="adagrad", lr=0.05, eps=1e-8,
             bag=("poisson", 5.0), key_space=100_000_000, preinsert=20_000_000,
             capacity=25_000_000, zipf_a=1.2),
    Workload(3, "streaming", B=65536, F=40, D=64, K=32, opt="adagrad", lr=0.05, eps=1e-8,
             bag=("poisson", 3.0), key_space=0, preinsert=1_000_000, capacity=52_000_000,
             zipf_a=1.1, p_new=0.0306, steps=200),
    Workload(4, "large_table", B=131072, F=200, D=64, K=64, opt="adagrad", lr=0.05, eps=1e-8,
             bag=("poisson", 4.0), key_space=300_000_000, preinsert=300_000_000,
             capacity=300_000_000, zipf_a=1.05, uniform_mix=0.5, key_bits=63),
]


def workload(index: int, scale: float = 1.0, **overrides) -> Workload:
    """Configuration ``index`` of the benchmark list; ``scale`` < 1 shrinks batch and table.

    Shrinking keeps F, D, K, the bag-length law and the popularity law, and scales B, the key
    space, the pre-inserted head and the capacity, so a shrunken workload has the same
    duplicate structure per sample at a size the CPU oracle finishes in seconds.
    """
    w = _FULL[index]
    if scale != 1.0:
        def s(v, lo=1):
            return max(lo, int(round(v * scale)))
        w = replace(w, B=s(w.B, 4), key_space=s(w.key_space, 64) if w.key_space else 0,
                    preinsert=s(w.preinsert, 32), capacity=s(w.capacity, 256))
        if w.p_new:
            w = replace(w, capacity=max(w.capacity, w.preinsert + 4 * int(w.B * w.F * w.mean_bag() * w.p_new) + 64))
    if overrides:
        w = replace(w, **overrides)
    return w


def zipf_truncated(rng: np.random.Generator, a: float, n_max: int, size: int) -> np.ndarray:
    """Ranks in [1, n_max] with P(r) proportional to r^-a: unbounded Zipf draws, re-drawn while
    they fall outside the support (exact rejection, acceptance >= 60 % for every workload)."""
    out = rng.zipf(a, size).astype(np.int64)
    bad = np.flatnonzero((out > n_max) | (out < 1))
    while bad.size:
        out[bad] = rng.zipf(a, bad.size)
        bad = bad[(out[bad] > n_max) | (out[bad] < 1)]
    return out


def bag_lengths(rng: np.random.Generator, w: Workload) -> np.ndarray:
    n = w.B * w.F
    kind = w.bag[0]
    if kind == "const":
        return np.full(n, int(w.bag[1]), dtype=np.int64)
    if kind == "uniform":
        return rng.integers(int(w.bag[1]), int(w.bag[2]) + 1, size=n, dtype=np.int64)
    if kind == "poisson":  # max(1, Poisson(lam)), not zero-truncated
        return np.maximum(1, rng.poisson(float(w.bag[1]), size=n)).astype(np.int64)
    raise ValueError(kind)


@dataclass
class Batch:
    B: int
    F: int
    keys: np.ndarray        # [nnz] uint64
    offsets: np.ndarray     # [B*F+1] int32; bag (b,f) = entries offsets[b*F+f] .. offsets[b*F+f+1]
    vals: Optional[np.ndarray] = None   # [nnz] float32 feature values; None => all ones
    labels: Optional[np.ndarray] = None  # [B] float32 in {0,1}
    ranks: Optional[np.ndarray] = None   # [nnz] int64 popularity rank of each entry (non-streaming workloads)

    @property
    def nnz(self) -> int:
        return int(self.keys.shape[0])


def _step_rng(w: Workload, step: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([w.seed, stream, step])))


def preinsert_keys(w: Workload, lo: int = 0, hi: Optional[int] = None) -> np.ndarray:
    """IDs of ranks lo+1 .. hi (default: the whole pre-inserted head), in rank order."""
    hi = w.preinsert if hi is None else hi
    return w.rank_to_key(np.arange(lo + 1, hi + 1, dtype=np.uint64))


def host_values(w: Workload, n: int, D: Optional[int] = None) -> np.ndarray:
    """[n, D+1] float32 initial weights N(0, init_std^2): D latent columns then the LR weight."""
    D = w.D if D is None else D
    rng = _step_rng(w, 0, stream=7)
    return (rng.standard_normal((n, D + 1)) * w.init_std).astype(np.float32)


def gen_batch(w: Workload, step: int = 0, with_vals: bool = False) -> Batch:
    """Batch ``step`` of a non-streaming workload (indices 0, 1, 2, 4)."""
    if w.p_new:
        raise ValueError("streaming workloads are generated by StreamingGenerator")
    rng = _step_rng(w, step, stream=1)
    lens = bag_lengths(rng, w)
    offsets = np.zeros(w.B * w.F + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    nnz = int(offsets[-1])
    if nnz >= 2**31:
        raise ValueError("batch too large for int32 offsets")
    if w.zipf_a is None:
        ranks = rng.integers(1, w.key_space + 1, size=nnz, dtype=np.int64)
    else:
        if w.uniform_mix > 0.0:
            uni = rng.random(nnz) < w.uniform_mix
            n_uni = int(uni.sum())
            ranks = np.empty(nnz, dtype=np.int64)
            ranks[uni] = rng.integers(1, w.preinsert + 1, size=n_uni, dtype=np.int64)
            ranks[~uni] = zipf_truncated(rng, w.zipf_a, w.key_space, nnz - n_uni)
        else:
            ranks = zipf_truncated(rng, w.zipf_a, w.key_space, nnz)
    keys = w.rank_to_key(ranks.astype(np.uint64))
    vals = None
    if with_vals:
        vals = rng.uniform(0.25, 2.0, size=nnz).astype(np.float32)
    labels = (rng.random(w.B) < 0.2).astype(np.float32)
    return Batch(w.B, w.F, keys, offsets.astype(np.int32), vals, labels, ranks)


class StreamingGenerator:
    """Streaming workload: each entry is a brand-new random 64-bit ID with probability
    ``p_new``, else the ID of an existing row drawn by popularity over the rows known so far.

    The generator mirrors the table's row -> key map on the host.  It relies only on the
    documented row-assignment rule of the table interface (the unseen distinct IDs of one call
    get consecutive rows in the order of their first occurrence); it does not look at the table.
    """

    _PERM_MULT = 2_654_435_761  # odd; rank -> row through (rank * mult) mod n_rows

    def __init__(self, w: Workload):
        if not w.p_new:
            raise ValueError("not a streaming workload")
        self.w = w
        self.step = 0
        self.row_keys = scramble64(np.arange(1, w.preinsert + 1, dtype=np.uint64))   # distinct: rows 0..preinsert-1
        self._known_sorted = np.sort(self.row_keys)

    def initial_keys(self) -> np.ndarray:
        return self.row_keys.copy()

    def grow_to(self, n_rows: int) -> np.ndarray:
        """Jumps to a later state of the stream without generating the steps in between: appends seeded
        random distinct IDs until `n_rows` rows are known and returns the appended IDs in row order (the
        caller inserts them into the table in this order, in one or several calls)."""
        rng = _step_rng(self.w, int(n_rows), stream=9)
        added = np.empty(0, dtype=np.uint64)
        while self.row_keys.shape[0] + added.shape[0] < n_rows:
            need = n_rows - self.row_keys.shape[0] - added.shape[0]
            cand = rng.integers(0, 2**64 - 1, size=need + need // 64 + 16, dtype=np.uint64)
            # distinct, unseen, in order of first occurrence
            u, first = np.unique(cand, return_index=True)
            cand = u[np.argsort(first, kind="stable")]
            for known in (self._known_sorted, np.sort(added)):
                if known.size:
                    pos = np.minimum(np.searchsorted(known, cand), known.shape[0] - 1)
                    cand = cand[known[pos] != cand]
            added = np.concatenate([added, cand[:need]])
        self.row_keys = np.concatenate([self.row_keys, added])
        self._known_sorted = np.sort(self.row_keys)
        return added

    def next_batch(self, p_new: Optional[float] = None) -> Batch:
        """The next batch; `p_new` overrides the workload's probability of a brand-new ID for this batch."""
        w = self.w
        p_new = w.p_new if p_new is None else float(p_new)
        rng = _step_rng(w, self.step, stream=1)
        lens = bag_lengths(rng, w)
        offsets = np.zeros(w.B * w.F + 1, dtype=np.int64)
        np.cumsum(lens, out=offsets[1:])
        nnz = int(offsets[-1])
        n_rows = self.row_keys.shape[0]
        ranks = zipf_truncated(rng, w.zipf_a, n_rows, nnz)
        rows = (ranks * self._PERM_MULT) % n_rows
        keys = self.row_keys[rows]
        fresh = rng.random(nnz) < p_new
        n_fresh = int(fresh.sum())
        keys[fresh] = rng.integers(0, 2**64 - 1, size=n_fresh, dtype=np.uint64)  # excludes the reserved ID
        # mirror of the table: unseen distinct IDs become new rows in order of first occurrence
        cand, first = np.unique(keys[fresh], return_index=True)
        known = self._known_sorted
        pos = np.minimum(np.searchsorted(known, cand), known.shape[0] - 1)
        unseen = known[pos] != cand
        add = cand[unseen][np.argsort(first[unseen], kind="stable")]
        self.row_keys = np.concatenate([self.row_keys, add])
        self._known_sorted = np.sort(self.row_keys)
        labels = (rng.random(w.B) < 0.2).astype(np.float32)
        self.step += 1
        return Batch(w.B, w.F, keys, offsets.astype(np.int32), None, labels)


def upstream_gradients(w: Workload, step: int = 0, pool: bool = True):
    """Seeded random upstream gradients of the shapes the backward pass takes
    (g_lr[B], g_fm[B], g_pool[B,F,D]), with the 1/B magnitude of a mean log-loss head."""
    rng = _step_rng(w, step, stream=3)
    g_lr = (rng.standard_normal(w.B) / w.B).astype(np.float32)
    g_fm = (rng.standard_normal(w.B) / w.B).astype(np.float32)
    g_pool = None
    if pool:
        g_pool = (rng.standard_normal((w.B, w.F, w.D), dtype=np.float32) / np.float32(w.B)).astype(np.float32)
    return g_lr, g_fm, g_pool


def head_weights(w: Workload) -> np.ndarray:
    """Fixed (untrained) [F, D] read-out of the pooled embeddings used by the tiny loss head."""
    rng = _step_rng(w, 0, stream=5)
    return (rng.standard_normal((w.F, w.D)) / np.sqrt(w.F * w.D)).astype(np.float32)


def dnn_layer_inputs(seed: int, B: int, F: int, D: int, H: int):
    """Inputs of the first fully-connected layer at the magnitudes training sees: pooled embeddings
    pool[B,F,D] ~ N(0, 0.05^2) (a few initialised rows summed), weights W[F*D,H] ~ N(0, 1/(F*D))
    (fan-in scaling) and an upstream gradient dY[B,H] ~ N(0, 0.01^2)."""
    rng = np.random.default_rng((int(seed), 0xD77))
    pool = (0.05 * rng.standard_normal((B, F, D), dtype=np.float32)).astype(np.float32)
    W = (rng.standard_normal((F * D, H), dtype=np.float32) / np.float32(np.sqrt(F * D))).astype(np.float32)
    dY = (0.01 * rng.standard_normal((B, H), dtype=np.float32)).astype(np.float32)
    return pool, W, dY


def tower_init(seed: int, F: int, D: int, hidden=(256, 128)):
    """Initial dense parameters of the tower after the pooled embeddings, for hidden widths H1..Hn:
    W1[F*D,H1], b1[H1], W2[H1,H2], b2[H2], ..., w_out[Hn], b0[1].  Weights N(0, 2/fan_in) (the usual
    scaling before a ReLU), hidden biases 0.01, output bias 0."""
    rng = np.random.default_rng((int(seed), 0x70E))
    n = lambda rows, cols: (rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(np.sqrt(2.0 / rows)))
    out, fan_in = {}, F * D
    for i, h in enumerate(hidden):
        out[f"W{i + 1}"] = n(fan_in, h)
        out[f"b{i + 1}"] = np.full(h, 0.01, np.float32)
        fan_in = h
    out["w_out"] = rng.standard_normal(fan_in, dtype=np.float32) * np.float32(np.sqrt(1.0 / fan_in))
    out["b0"] = np.zeros(1, np.float32)
    return out


def cross_init(seed: int, F: int, D: int, n_cross: int = 2):
    """Initial parameters of a DCN cross network over d = F*D columns: cw{l}[d] ~ N(0, 1/d) and cb{l}[d] = 0 for
    l = 1..n_cross, and w_cross[d] ~ N(0, 1/d), the output unit's weights on the network's result."""
    rng = np.random.default_rng((int(seed), 0xC705))
    d = F * D
    out = {}
    for l in range(1, n_cross + 1):
        out[f"cw{l}"] = rng.standard_normal(d, dtype=np.float32) * np.float32(np.sqrt(1.0 / d))
        out[f"cb{l}"] = np.zeros(d, np.float32)
    out["w_cross"] = rng.standard_normal(d, dtype=np.float32) * np.float32(np.sqrt(1.0 / d))
    return out


def planted_labels(batch: Batch, seed: int, base_rate_logit: float = -1.4, strength: float = 1.5) -> np.ndarray:
    """Click labels a model can learn from the IDs: every ID carries a hidden weight in [-1,1)
    (a scramble of the ID, centred on the batch's entry mean so that hot IDs do not shift every
    sample alike), a sample's score is the sum of its entries' hidden weights over sqrt(n), n its
    number of entries, and y ~ Bernoulli(sigmoid(base_rate_logit + strength * score))."""
    hidden = (scramble64(batch.keys ^ np.uint64(0x5EEDF00D ^ int(seed))) >> np.uint64(11)).astype(np.float64)
    hidden = hidden / float(1 << 52) - 1.0
    hidden -= hidden.mean() if hidden.size else 0.0
    ends = batch.offsets[batch.F::batch.F].astype(np.int64)
    starts = batch.offsets[0:-1:batch.F].astype(np.int64)
    csum = np.concatenate([[0.0], np.cumsum(hidden)])
    n = np.maximum(ends - starts, 1)
    score = (csum[ends] - csum[starts]) / np.sqrt(n)
    p = 1.0 / (1.0 + np.exp(-(base_rate_logit + strength * score)))
    rng = np.random.default_rng((int(seed), 0x1AB, int(batch.keys.shape[0])))
    return (rng.random(batch.B) < p).astype(np.float32)
