"""ctypes front-end of the CPU oracle (``des_oracle.c``).

TEST INFRASTRUCTURE ONLY: importable from ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``; never from the HIP path.  Everything here is argument
marshalling; the arithmetic is in the C file, in double precision.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "des_oracle.c")
_LIB = os.path.join(_HERE, "libdes_oracle.so")

SHARD_KEY_HASH, SHARD_FIELD_MOD = 0, 1
OPT_NONE, OPT_SGD, OPT_ADAGRAD, OPT_ADAM, OPT_FTRL = 0, 1, 2, 3, 4
OK, ERR_INVALID_ARG, ERR_INVALID_KEY, ERR_FULL = 0, 1, 2, 3


_LIB_OMP = os.path.join(_HERE, "libdes_oracle_omp.so")


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, no FMA contraction so fp32 steps round as written): the plain
    single-threaded library every test uses, and a second one with -fopenmp for the all-cores leg of the
    benchmark's CPU baseline (same source, the marked loops split over threads)."""
    for path, extra in ((_LIB, []), (_LIB_OMP, ["-fopenmp"])):
        if force or not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_SRC):
            subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-std=c11", "-shared", "-fPIC", *extra,
                                   "-o", path, _SRC, "-lm"])
    return _LIB


class Optimizer(C.Structure):
    """Mirror of the C struct oracle_optimizer."""
    _fields_ = [("opt_emb", C.c_int32), ("opt_w", C.c_int32), ("lr", C.c_float), ("eps", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("step", C.c_int64),
                ("ftrl_alpha", C.c_float), ("ftrl_beta", C.c_float), ("ftrl_l1", C.c_float), ("ftrl_l2", C.c_float)]


_LIB_UBSAN = os.path.join(_HERE, "libdes_oracle_ubsan.so")


def build_ubsan() -> str:
    """A third build with gcc's undefined-behaviour sanitizer (signed overflow, bad shifts, misaligned or
    out-of-bounds accesses it can see, ...), every finding fatal.  Used by one test, which runs the oracle's
    whole interface through it in a child process (DES_ORACLE_LIB selects the library to load)."""
    subprocess.check_call(["gcc", "-O1", "-g", "-ffp-contract=off", "-std=c11", "-shared", "-fPIC",
                           "-fsanitize=undefined", "-fno-sanitize-recover=all", "-o", _LIB_UBSAN, _SRC, "-lm"])
    return _LIB_UBSAN


_lib = None
_use_openmp = False


def use_openmp(on: bool) -> int:
    """Switch every later call to the OpenMP build (or back); tables created before the switch must not be
    used after it.  Returns the number of threads the selected build runs on."""
    global _lib, _use_openmp
    if bool(on) != _use_openmp:
        _use_openmp, _lib = bool(on), None
    return int(lib().oracle_threads())


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(os.environ.get("DES_ORACLE_LIB") or (_LIB_OMP if _use_openmp else _LIB))
        L.oracle_threads.restype = C.c_int; L.oracle_threads.argtypes = []
        vp, i32, i64, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float
        L.oracle_mix64.restype = u64; L.oracle_mix64.argtypes = [u64]
        L.oracle_shard.restype = C.c_int; L.oracle_shard.argtypes = [u64, i32, C.c_int, C.c_int]
        L.oracle_init_value.restype = f32; L.oracle_init_value.argtypes = [u64, C.c_int, u64, f32]
        L.oracle_table_create.restype = vp; L.oracle_table_create.argtypes = [C.c_int, i64, u64, f32]
        L.oracle_table_destroy.restype = None; L.oracle_table_destroy.argtypes = [vp]
        L.oracle_table_size.restype = i64; L.oracle_table_size.argtypes = [vp]
        for name in ("row_keys", "emb", "w", "acc_emb", "acc_w", "acc2_emb", "acc2_w"):
            fn = getattr(L, "oracle_table_" + name); fn.restype = vp; fn.argtypes = [vp]
        L.oracle_table_insert.restype = C.c_int; L.oracle_table_insert.argtypes = [vp, vp, i64, vp, vp]
        L.oracle_table_find.restype = C.c_int; L.oracle_table_find.argtypes = [vp, vp, i64, C.c_int, vp]
        L.oracle_partial_forward.restype = None
        L.oracle_partial_forward.argtypes = [vp, i64, i32, vp, vp, vp, vp, C.c_int, C.c_int, vp, vp, vp, vp]
        L.oracle_aggregate.restype = None; L.oracle_aggregate.argtypes = [vp, C.c_int, i64, vp]
        L.oracle_fm_finalize.restype = None; L.oracle_fm_finalize.argtypes = [vp, vp, i64, C.c_int, vp]
        L.oracle_backward_update.restype = i64
        L.oracle_backward_update.argtypes = [vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, C.c_int, f32, f32,
                                             vp, vp, vp, vp]
        L.oracle_backward_update_opt.restype = i64
        L.oracle_backward_update_opt.argtypes = [vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, C.POINTER(Optimizer),
                                                 vp, vp, vp, vp]
        L.oracle_dnn_partial_forward.restype = None
        L.oracle_dnn_partial_forward.argtypes = [vp, vp, i64, i32, C.c_int, C.c_int, C.c_int, vp]
        L.oracle_dnn_backward.restype = None
        L.oracle_dnn_backward.argtypes = [vp, vp, vp, i64, i32, C.c_int, C.c_int, vp, vp]
        L.oracle_cross_partial.restype = None
        L.oracle_cross_partial.argtypes = [vp, vp, i64, i32, C.c_int, C.c_int, vp]
        L.oracle_cross_apply.restype = None; L.oracle_cross_apply.argtypes = [vp, vp, vp, vp, i64, i64, vp]
        L.oracle_cross_partial_backward.restype = None
        L.oracle_cross_partial_backward.argtypes = [vp, vp, vp, i64, i64, vp, vp]
        L.oracle_cross_backward.restype = None
        L.oracle_cross_backward.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp, vp]
        L.oracle_bias_act.restype = None; L.oracle_bias_act.argtypes = [vp, vp, i64, C.c_int, C.c_int, vp]
        L.oracle_bias_act_backward.restype = None
        L.oracle_bias_act_backward.argtypes = [vp, vp, i64, C.c_int, C.c_int, vp, vp]
        L.oracle_head.restype = None
        L.oracle_head.argtypes = [vp, vp, vp, vp, f32, vp, i64, C.c_int, vp, vp, vp, vp, vp, vp, vp]
        L.oracle_dense_update.restype = None
        L.oracle_dense_update.argtypes = [vp, vp, vp, vp, i64, C.POINTER(Optimizer)]
        L.oracle_table_migrate.restype = vp; L.oracle_table_migrate.argtypes = [vp, vp, i64]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def mix64(z: int) -> int:
    return int(lib().oracle_mix64(C.c_uint64(int(z) & 0xFFFFFFFFFFFFFFFF)))


def shard(key: int, field: int, K: int, policy: int = SHARD_KEY_HASH) -> int:
    return int(lib().oracle_shard(C.c_uint64(int(key)), int(field), int(K), int(policy)))


def init_value(key: int, column: int, seed: int, init_scale: float) -> float:
    return float(lib().oracle_init_value(C.c_uint64(int(key)), int(column), C.c_uint64(int(seed)),
                                         C.c_float(init_scale)))


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle status {code}")
        self.code = code


class Table:
    """Key -> row map plus fp32 weights and optimizer state; see ``des_oracle.c``."""

    def __init__(self, D: int, capacity: int, seed: int = 0, init_scale: float = 0.01):
        self.D, self.capacity = int(D), int(capacity)
        self._h = lib().oracle_table_create(self.D, self.capacity, C.c_uint64(seed), C.c_float(init_scale))
        if not self._h:
            raise OracleError(ERR_INVALID_ARG)

    def close(self):
        if self._h:
            lib().oracle_table_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def n_rows(self) -> int:
        return int(lib().oracle_table_size(self._h))

    def _view(self, name, ctype, shape):
        ptr = getattr(lib(), "oracle_table_" + name)(self._h)
        n = int(np.prod(shape))
        if n == 0:
            return np.zeros(shape, dtype=np.dtype(ctype))
        return np.ctypeslib.as_array(C.cast(ptr, C.POINTER(ctype)), shape=(n,)).reshape(shape)

    # views of the live rows (no copy)
    @property
    def row_keys(self): return self._view("row_keys", C.c_uint64, (self.n_rows,))
    @property
    def emb(self): return self._view("emb", C.c_float, (self.n_rows, self.D))
    @property
    def w(self): return self._view("w", C.c_float, (self.n_rows,))
    @property
    def acc_emb(self): return self._view("acc_emb", C.c_float, (self.n_rows, self.D))
    @property
    def acc_w(self): return self._view("acc_w", C.c_float, (self.n_rows,))
    @property
    def acc2_emb(self): return self._view("acc2_emb", C.c_float, (self.n_rows, self.D))
    @property
    def acc2_w(self): return self._view("acc2_w", C.c_float, (self.n_rows,))

    def migrate(self, keep=None, new_capacity: Optional[int] = None) -> "Table":
        """New table holding the rows r with keep[r] != 0 (all when keep is None), renumbered in
        ascending old-row order, weights and optimizer state unchanged; capacity `new_capacity`."""
        cap = self.capacity if new_capacity is None else int(new_capacity)
        keep = None if keep is None else _c(np.asarray(keep) != 0, np.uint8)
        if keep is not None and keep.shape[0] != self.n_rows:
            raise ValueError("keep must have one flag per row")
        h = lib().oracle_table_migrate(self._h, _p(keep), cap)
        if not h:
            raise OracleError(ERR_FULL)
        t = Table.__new__(Table)
        t.D, t.capacity, t._h = self.D, cap, h
        return t

    def insert(self, keys, values=None) -> np.ndarray:
        keys = _c(keys, np.uint64)
        values = _c(values, np.float32)
        if values is not None and values.shape != (keys.shape[0], self.D + 1):
            raise ValueError("values must be [n, D+1]")
        rows = np.empty(keys.shape[0], dtype=np.int32)
        rc = lib().oracle_table_insert(self._h, _p(keys), keys.shape[0], _p(values), _p(rows))
        if rc:
            raise OracleError(rc)
        return rows

    def find(self, keys, insert_missing: bool = False) -> np.ndarray:
        keys = _c(keys, np.uint64)
        rows = np.empty(keys.shape[0], dtype=np.int32)
        rc = lib().oracle_table_find(self._h, _p(keys), keys.shape[0], int(insert_missing), _p(rows))
        if rc:
            raise OracleError(rc)
        return rows

    def partial_forward(self, B, F, keys, offsets, rows, K, policy=SHARD_KEY_HASH, vals=None,
                        lr=True, fm=True, pool=True):
        """Double-precision partials: dict with P_lr[K,B], P_sum[K,B,D], P_sq[K,B], P_pool[K,B,F,D]."""
        keys, offsets, rows = _c(keys, np.uint64), _c(offsets, np.int32), _c(rows, np.int32)
        vals = _c(vals, np.float32)
        D = self.D
        out = {
            "P_lr": np.empty((K, B), np.float64) if lr else None,
            "P_sum": np.empty((K, B, D), np.float64) if fm else None,
            "P_sq": np.empty((K, B), np.float64) if fm else None,
            "P_pool": np.empty((K, B, F, D), np.float64) if pool else None,
        }
        lib().oracle_partial_forward(self._h, B, F, _p(keys), _p(offsets), _p(vals), _p(rows), K, policy,
                                     _p(out["P_lr"]), _p(out["P_sum"]), _p(out["P_sq"]), _p(out["P_pool"]))
        return out

    def backward_update(self, B, F, offsets, rows, g_lr=None, g_fm=None, A_sum=None, g_pool=None,
                        opt=OPT_NONE, lr=0.0, eps=0.0, vals=None, optimizer: Optional[Optimizer] = None):
        """Merge duplicate-row gradients (ascending row order) and apply the optimizer in place
        (`optimizer` selects separate optimizers for latent vectors and LR weights; otherwise
        `opt`, `lr`, `eps` apply to both).  Returns dict(uniq_rows, uniq_keys, counts,
        merged[U,D+1] float64)."""
        offsets, rows = _c(offsets, np.int32), _c(rows, np.int32)
        vals = _c(vals, np.float32)
        g_lr, g_fm, A_sum, g_pool = (_c(a, np.float32) for a in (g_lr, g_fm, A_sum, g_pool))
        if (g_fm is None) != (A_sum is None):
            raise ValueError("g_fm and A_sum go together")
        nnz = int(offsets[B * F])
        uniq_rows = np.empty(nnz, np.int32); uniq_keys = np.empty(nnz, np.uint64)
        counts = np.empty(nnz, np.int32); merged = np.empty((nnz, self.D + 1), np.float64)
        if optimizer is not None:
            U = int(lib().oracle_backward_update_opt(self._h, B, F, _p(offsets), _p(vals), _p(rows), _p(g_lr),
                                                     _p(g_fm), _p(A_sum), _p(g_pool), C.byref(optimizer),
                                                     _p(uniq_rows), _p(uniq_keys), _p(counts), _p(merged)))
        else:
            U = int(lib().oracle_backward_update(self._h, B, F, _p(offsets), _p(vals), _p(rows), _p(g_lr), _p(g_fm),
                                                 _p(A_sum), _p(g_pool), opt, C.c_float(lr), C.c_float(eps),
                                                 _p(uniq_rows), _p(uniq_keys), _p(counts), _p(merged)))
        return {"uniq_rows": uniq_rows[:U].copy(), "uniq_keys": uniq_keys[:U].copy(),
                "counts": counts[:U].copy(), "merged": merged[:U].copy()}


def aggregate(P: np.ndarray) -> np.ndarray:
    """Sum over the leading (shard) axis in double: the on-device stand-in of the collective."""
    P = np.ascontiguousarray(P, dtype=np.float64)
    K = P.shape[0]
    n = int(np.prod(P.shape[1:]))
    out = np.empty(P.shape[1:], np.float64)
    lib().oracle_aggregate(_p(P), K, n, _p(out))
    return out


def fm_finalize(A_sum: np.ndarray, A_sq: np.ndarray) -> np.ndarray:
    A_sum = np.ascontiguousarray(A_sum, np.float64); A_sq = np.ascontiguousarray(A_sq, np.float64)
    B, D = A_sum.shape
    out = np.empty(B, np.float64)
    lib().oracle_fm_finalize(_p(A_sum), _p(A_sq), B, D, _p(out))
    return out


def dnn_partial_forward(pool: np.ndarray, W: np.ndarray, K: int) -> np.ndarray:
    """Per-shard partials Y_partial[K,B,H] (float64) of the first fully-connected layer; pool is
    [B,F,D] fp32, W is [F*D,H] fp32, shard of field f is f mod K."""
    pool, W = _c(pool, np.float32), _c(W, np.float32)
    B, F, D = pool.shape
    H = W.shape[1]
    if W.shape[0] != F * D:
        raise ValueError("W must be [F*D, H]")
    out = np.empty((K, B, H), np.float64)
    lib().oracle_dnn_partial_forward(_p(pool), _p(W), B, F, D, H, K, _p(out))
    return out


def dnn_backward(pool: np.ndarray, W: np.ndarray, dY: np.ndarray, want_g_pool: bool = True, want_dW: bool = True):
    """(g_pool[B,F,D], dW[F*D,H]) in float64 for the upstream gradient dY[B,H] of the aggregate
    (None for an output that is not wanted)."""
    pool, W, dY = _c(pool, np.float32), _c(W, np.float32), _c(dY, np.float32)
    B, F, D = pool.shape
    H = W.shape[1]
    if W.shape[0] != F * D or dY.shape != (B, H):
        raise ValueError("shape mismatch")
    g_pool = np.empty((B, F, D), np.float64) if want_g_pool else None
    dW = np.empty((F * D, H), np.float64) if want_dW else None
    lib().oracle_dnn_backward(_p(pool), _p(W), _p(dY), B, F, D, H, _p(g_pool), _p(dW))
    return g_pool, dW


def cross_partial(xl: np.ndarray, w: np.ndarray, K: int) -> np.ndarray:
    """Per-shard scalars P[K,B] (float64) of a DCN cross layer: xl is [B,F,D] fp32, w is [F*D] fp32, the
    columns of field f belong to shard f mod K."""
    xl, w = _c(xl, np.float32), _c(w, np.float32)
    B, F, D = xl.shape
    if w.shape != (F * D,):
        raise ValueError("w must be [F*D]")
    out = np.empty((K, B), np.float64)
    lib().oracle_cross_partial(_p(xl), _p(w), B, F, D, K, _p(out))
    return out


def cross_partial_backward(xl: np.ndarray, w: np.ndarray, g_s: np.ndarray):
    """(g_xl, dw[d]) in float64 for a gradient g_s[B] of the aggregated scalar xl w."""
    xl, w, g_s = _c(xl, np.float32), _c(w, np.float32), _c(g_s, np.float32)
    B, d = xl.shape[0], w.shape[0]
    if xl.size != B * d or g_s.shape != (B,):
        raise ValueError("shape mismatch")
    g_xl, dw = np.empty(xl.shape, np.float64), np.empty(d, np.float64)
    lib().oracle_cross_partial_backward(_p(xl), _p(w), _p(g_s), B, d, _p(g_xl), _p(dw))
    return g_xl, dw


def cross_apply(x0: np.ndarray, xl: np.ndarray, s: np.ndarray, bias: np.ndarray) -> np.ndarray:
    """y[B,d] = x0 * s[:,None] + bias + xl in float64; s is the aggregated scalar per sample (fp32)."""
    x0, xl, s, bias = _c(x0, np.float32), _c(xl, np.float32), _c(s, np.float32), _c(bias, np.float32)
    B = x0.shape[0]
    d = x0.size // max(B, 1)
    if xl.shape != x0.shape or s.shape != (B,) or bias.shape != (d,):
        raise ValueError("shape mismatch")
    y = np.empty(x0.shape, np.float64)
    lib().oracle_cross_apply(_p(x0), _p(xl), _p(s), _p(bias), B, d, _p(y))
    return y


def cross_backward(x0: np.ndarray, xl: np.ndarray, w: np.ndarray, s: np.ndarray, g_y: np.ndarray):
    """(g_s[B], g_xl, g_x0, dw[d], db[d]) in float64 for the upstream gradient g_y of the layer's output;
    g_x0 is this layer's share of the gradient of x0."""
    x0, xl, w, s, g_y = (_c(a, np.float32) for a in (x0, xl, w, s, g_y))
    B = x0.shape[0]
    d = w.shape[0]
    if xl.shape != x0.shape or g_y.shape != x0.shape or x0.size != B * d or s.shape != (B,):
        raise ValueError("shape mismatch")
    g_s = np.empty(B, np.float64)
    g_xl, g_x0 = np.empty(x0.shape, np.float64), np.empty(x0.shape, np.float64)
    dw, db = np.empty(d, np.float64), np.empty(d, np.float64)
    lib().oracle_cross_backward(_p(x0), _p(xl), _p(w), _p(s), _p(g_y), B, d, _p(g_s), _p(g_xl), _p(g_x0), _p(dw), _p(db))
    return g_s, g_xl, g_x0, dw, db


def bias_act(Z: np.ndarray, bias: Optional[np.ndarray], relu: bool) -> np.ndarray:
    """A = relu(Z + bias) (or Z + bias) in float64; Z is [B,H] float64 (an aggregate)."""
    Z = _c(Z, np.float64); bias = _c(bias, np.float32)
    B, H = Z.shape
    A = np.empty((B, H), np.float64)
    lib().oracle_bias_act(_p(Z), _p(bias), B, H, int(relu), _p(A))
    return A


def bias_act_backward(A: np.ndarray, dA: np.ndarray, relu: bool):
    """(dZ[B,H], dbias[H]) in float64 from the fp32 forward output A and upstream gradient dA."""
    A, dA = _c(A, np.float32), _c(dA, np.float32)
    B, H = A.shape
    dZ = np.empty((B, H), np.float64); dbias = np.empty(H, np.float64)
    lib().oracle_bias_act_backward(_p(A), _p(dA), B, H, int(relu), _p(dZ), _p(dbias))
    return dZ, dbias


def head(labels: np.ndarray, A_lr=None, fm2=None, a=None, w_out=None, b0: float = 0.0):
    """Output unit + mean log-loss + gradients; dict(logit, p, loss, g_logit, da, dw_out, db0), float64."""
    labels = _c(labels, np.float32)
    A_lr, fm2, a, w_out = (_c(x, np.float32) for x in (A_lr, fm2, a, w_out))
    B = labels.shape[0]
    H = 0 if a is None else a.shape[1]
    if (a is None) != (w_out is None):
        raise ValueError("a and w_out go together")
    out = {"logit": np.empty(B), "p": np.empty(B), "g_logit": np.empty(B),
           "da": None if a is None else np.empty((B, H)), "dw_out": None if a is None else np.empty(H)}
    loss, db0 = C.c_double(0.0), C.c_double(0.0)
    lib().oracle_head(_p(A_lr), _p(fm2), _p(a), _p(w_out), C.c_float(b0), _p(labels), B, H, _p(out["logit"]),
                      _p(out["p"]), C.byref(loss), _p(out["g_logit"]), _p(out["da"]), _p(out["dw_out"]), C.byref(db0))
    out["loss"], out["db0"] = loss.value, db0.value
    return out


def dense_update(theta: np.ndarray, grad: np.ndarray, optimizer: Optimizer, s1=None, s2=None):
    """In-place optimizer step (optimizer.opt_emb) on fp32 arrays theta (and state s1, s2)."""
    for x in (theta, s1, s2):
        if x is not None and not (x.dtype == np.float32 and x.flags.c_contiguous):
            raise ValueError("theta and state must be contiguous float32 (updated in place)")
    grad = _c(grad, np.float32)
    lib().oracle_dense_update(_p(theta), _p(grad), _p(s1), _p(s2), theta.size, C.byref(optimizer))


def mark_seen(last_seen: np.ndarray, rows: np.ndarray, stamp: int) -> None:
    """Least-recently-seen bookkeeping, the definition written out: every row that occurs in `rows`
    (entries with row -1 are absent keys) gets `stamp`; in place on a uint32 array."""
    rows = np.asarray(rows)
    last_seen[rows[rows >= 0]] = np.uint32(stamp)


def select_recent(last_seen: np.ndarray, n_rows: int, min_stamp: int) -> np.ndarray:
    """keep[r] = last_seen[r] >= min_stamp for the first n_rows rows."""
    return (np.asarray(last_seen[:n_rows]) >= np.uint32(min_stamp)).astype(np.uint8)
