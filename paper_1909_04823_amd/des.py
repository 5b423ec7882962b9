"""ctypes binding of libdes.so: same names as the C interface (include/des.h), argument
marshalling only.  PyTorch supplies device memory (tensors) and the current HIP stream; every
step of the path runs in the library's kernels.  Importing this module fails loudly when the
library has not been built (python -m paper_1909_04823_amd.build)."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdes.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1909_04823_amd.build`; "
                      "there is no fallback path")
_lib = C.CDLL(LIB_PATH)

OK, ERR_INVALID_ARG, ERR_INVALID_KEY, ERR_FULL, ERR_WORKSPACE, ERR_DEVICE = range(6)
SHARD_KEY_HASH, SHARD_FIELD_MOD = 0, 1
OPT_NONE, OPT_SGD, OPT_ADAGRAD, OPT_ADAM, OPT_FTRL = 0, 1, 2, 3, 4
MISS_ZERO, MISS_INSERT = 0, 1

EXPORTS = [
    "des_table_query_bytes", "des_table_create", "des_table_destroy", "des_table_insert", "des_table_find",
    "des_table_size", "des_table_status", "des_table_clear_status", "des_table_export_keys", "des_partial_forward_lr", "des_partial_forward_fm",
    "des_partial_forward_pool", "des_partial_forward", "des_aggregate_partials", "des_aggregate_forward", "des_fm_finalize",
    "des_backward_update_sgd", "des_backward_update_adagrad", "des_backward_update", "des_backward_merge", "des_backward_prepare",
    "des_dnn_partial_forward", "des_dnn_backward_bytes", "des_dnn_backward",
    "des_batch_validate", "des_table_migrate_bytes", "des_table_migrate", "des_table_compact", "des_table_mark_seen", "des_table_select_recent",
    "des_aggregate_bias_act", "des_dense_workspace_bytes", "des_bias_act_backward", "des_bias_act_backward_static", "des_head", "des_dense_update",
    "des_cross_partial", "des_cross_apply", "des_cross_backward_bytes", "des_cross_backward", "des_cross_partial_backward",
    "des_cross_net_bytes", "des_cross_net_partial", "des_cross_net_forward", "des_cross_net_backward",
    "des_ceiling_gather_bytes", "des_ceiling_gather", "des_ceiling_update",
    "des_profile_enable", "des_profile_read", "des_status_string",
]


class TableConfig(C.Structure):
    _fields_ = [("dim", C.c_int32), ("capacity_rows", C.c_int64), ("num_shards", C.c_int32),
                ("shard_policy", C.c_int32), ("opt", C.c_int32), ("init_seed", C.c_uint64),
                ("init_scale", C.c_float), ("emb", C.c_void_p), ("w", C.c_void_p), ("acc_emb", C.c_void_p),
                ("acc_w", C.c_void_p), ("row_keys", C.c_void_p), ("slots", C.c_void_p), ("slots_bytes", C.c_size_t),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("acc2_emb", C.c_void_p), ("acc2_w", C.c_void_p)]


class BatchDesc(C.Structure):
    _fields_ = [("B", C.c_int64), ("F", C.c_int32), ("nnz", C.c_int64), ("keys", C.c_void_p),
                ("offsets", C.c_void_p), ("vals", C.c_void_p)]


class BackwardIO(C.Structure):
    _fields_ = [("g_lr", C.c_void_p), ("g_fm", C.c_void_p), ("A_sum", C.c_void_p), ("g_pool", C.c_void_p),
                ("uniq_rows_out", C.c_void_p), ("uniq_keys_out", C.c_void_p), ("counts_out", C.c_void_p),
                ("merged_out", C.c_void_p), ("n_uniq_out", C.c_void_p)]


class Optimizer(C.Structure):
    """des_optimizer_t"""
    _fields_ = [("opt_emb", C.c_int32), ("opt_w", C.c_int32), ("lr", C.c_float), ("eps", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("step", C.c_int64),
                ("ftrl_alpha", C.c_float), ("ftrl_beta", C.c_float), ("ftrl_l1", C.c_float), ("ftrl_l2", C.c_float)]


class KernelTime(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int64), ("total_ms", C.c_double)]


vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
_sig = {
    "des_table_query_bytes": [C.POINTER(TableConfig), i64, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)],
    "des_table_create": [C.POINTER(TableConfig), C.POINTER(vp)],
    "des_table_destroy": [vp],
    "des_table_insert": [vp, vp, i64, vp, vp, vp],
    "des_table_find": [vp, vp, i64, i32, vp, vp],
    "des_table_size": [vp, C.POINTER(i64)],
    "des_table_status": [vp],
    "des_table_clear_status": [vp],
    "des_table_export_keys": [vp, vp, i64, vp],
    "des_partial_forward_lr": [vp, C.POINTER(BatchDesc), vp, vp, vp],
    "des_partial_forward_fm": [vp, C.POINTER(BatchDesc), vp, vp, vp, vp],
    "des_partial_forward_pool": [vp, C.POINTER(BatchDesc), vp, vp, i32, vp],
    "des_partial_forward": [vp, C.POINTER(BatchDesc), vp, vp, vp, vp, vp, vp],
    "des_aggregate_partials": [vp, i32, i64, vp, vp],
    "des_fm_finalize": [vp, vp, i64, i32, vp, vp],
    "des_aggregate_forward": [vp, vp, vp, i32, i64, i32, vp, vp, vp, vp, vp],
    "des_backward_update_sgd": [vp, C.POINTER(BatchDesc), vp, C.POINTER(BackwardIO), f32, vp],
    "des_backward_update_adagrad": [vp, C.POINTER(BatchDesc), vp, C.POINTER(BackwardIO), f32, f32, vp],
    "des_backward_update": [vp, C.POINTER(BatchDesc), vp, C.POINTER(BackwardIO), C.POINTER(Optimizer), vp],
    "des_backward_merge": [vp, C.POINTER(BatchDesc), vp, C.POINTER(BackwardIO), vp],
    "des_backward_prepare": [vp, C.POINTER(BatchDesc), vp, vp],
    "des_dnn_partial_forward": [vp, vp, i64, i32, i32, i32, i32, vp, vp],
    "des_dnn_backward_bytes": [i64, i32, i32, i32, C.POINTER(C.c_size_t)],
    "des_dnn_backward": [vp, vp, vp, i64, i32, i32, i32, vp, vp, vp, C.c_size_t, vp],
    "des_aggregate_bias_act": [vp, i32, i64, i32, vp, i32, vp, vp],
    "des_dense_workspace_bytes": [i32, C.POINTER(C.c_size_t)],
    "des_bias_act_backward": [vp, vp, i64, i32, i32, vp, vp, vp, C.c_size_t, vp],
    "des_bias_act_backward_static": [vp, vp, i64, i32, i32, vp, vp, vp],
    "des_head": [vp, vp, vp, vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp],
    "des_dense_update": [vp, vp, vp, vp, i64, C.POINTER(Optimizer), vp],
    "des_batch_validate": [vp, C.POINTER(BatchDesc), vp, C.POINTER(i64), vp],
    "des_table_migrate_bytes": [i64, C.POINTER(C.c_size_t)],
    "des_table_migrate": [vp, vp, vp, vp, vp, C.POINTER(i64), vp],
    "des_table_compact": [vp, vp, vp, vp, C.c_size_t, C.POINTER(i64), vp],
    "des_table_mark_seen": [vp, i64, C.c_uint32, vp, vp],
    "des_table_select_recent": [vp, i64, C.c_uint32, vp, vp],
    "des_cross_partial": [vp, vp, i64, i32, i32, i32, vp, vp],
    "des_cross_apply": [vp, vp, vp, vp, i64, i64, vp, vp],
    "des_cross_backward_bytes": [i64, i64, C.POINTER(C.c_size_t)],
    "des_cross_backward": [vp, vp, vp, vp, vp, i64, i64, vp, vp, i32, vp, vp, vp, C.c_size_t, vp],
    "des_cross_partial_backward": [vp, vp, vp, i64, i64, vp, vp, vp, C.c_size_t, vp],
    "des_cross_net_bytes": [i64, i64, i32, C.POINTER(C.c_size_t)],
    "des_cross_net_partial": [vp, vp, i64, i32, i32, i32, i32, vp, vp],
    "des_cross_net_forward": [vp, vp, vp, i64, i64, i32, vp, vp, vp, C.c_size_t, vp],
    "des_cross_net_backward": [vp, vp, vp, vp, vp, vp, i64, i64, i32, vp, i32, vp, vp, vp, C.c_size_t, vp],
    "des_ceiling_gather_bytes": [C.POINTER(C.c_size_t)],
    "des_ceiling_gather": [vp, i32, i64, vp, i64, i64, vp, i64, vp, C.c_size_t, vp],
    "des_ceiling_update": [vp, vp, i32, i64, i64, vp, i64, vp],
    "des_profile_enable": [i32],
    "des_profile_read": [C.POINTER(KernelTime), i32, C.POINTER(i32)],
}
for _name, _args in _sig.items():
    _fn = getattr(_lib, _name)
    _fn.argtypes = _args
    _fn.restype = C.c_int
_lib.des_status_string.argtypes = [C.c_int]
_lib.des_status_string.restype = C.c_char_p


class DesError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = int(code)
        super().__init__(f"{where}: {_lib.des_status_string(self.code).decode()} (status {self.code})")


def _check(code: int, where: str):
    if code != OK:
        raise DesError(code, where)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


class Batch:
    """Device-resident CSR batch (keys int64 tensor holding the uint64 bit patterns)."""

    def __init__(self, B: int, F: int, keys: torch.Tensor, offsets: torch.Tensor, vals: Optional[torch.Tensor] = None):
        assert keys.dtype == torch.int64 and offsets.dtype == torch.int32
        assert offsets.numel() == B * F + 1
        assert vals is None or (vals.dtype == torch.float32 and vals.numel() == keys.numel())
        self.B, self.F, self.nnz = int(B), int(F), int(keys.numel())
        self.keys, self.offsets, self.vals = keys, offsets, vals
        self.desc = BatchDesc(self.B, self.F, self.nnz, _ptr(keys), _ptr(offsets), _ptr(vals))

    @staticmethod
    def from_numpy(b, device="cuda"):
        keys = torch.from_numpy(b.keys.view("int64")).to(device)
        offsets = torch.from_numpy(b.offsets).to(device)
        vals = None if b.vals is None else torch.from_numpy(b.vals).to(device)
        return Batch(b.B, b.F, keys, offsets, vals)


class Table:
    """Owns the tensors that back one table and the library handle."""

    def __init__(self, dim: int, capacity: int, num_shards: int = 1, shard_policy: int = SHARD_KEY_HASH,
                 opt: int = OPT_ADAGRAD, init_seed: int = 0, init_scale: float = 0.01, max_n: int = 1 << 20,
                 device="cuda", state_arrays=None):
        """`opt` decides which optimizer state arrays are allocated (Adagrad: one per weight,
        Adam: two, FTRL: two for the LR weight); `state_arrays=(n_emb, n_w)` overrides that for
        mixed settings such as Adagrad embeddings with FTRL order-1 weights (1, 2)."""
        self.dim, self.capacity, self.K = int(dim), int(capacity), int(num_shards)
        self.max_n = int(max_n)
        cfg = TableConfig()
        cfg.dim, cfg.capacity_rows, cfg.num_shards = self.dim, self.capacity, self.K
        cfg.shard_policy, cfg.opt, cfg.init_seed, cfg.init_scale = shard_policy, opt, init_seed, init_scale
        sb, wb = C.c_size_t(0), C.c_size_t(0)
        _check(_lib.des_table_query_bytes(C.byref(cfg), self.max_n, C.byref(sb), C.byref(wb)), "des_table_query_bytes")
        dev = torch.device(device)
        self.emb = torch.empty((self.capacity, self.dim), dtype=torch.float32, device=dev)
        self.w = torch.empty((self.capacity,), dtype=torch.float32, device=dev)
        # opt says which state arrays to allocate: ADAGRAD one per weight, ADAM two, FTRL two for the LR weight
        if state_arrays is None:
            n_emb = {OPT_ADAGRAD: 1, OPT_ADAM: 2}.get(opt, 0)
            n_w = {OPT_ADAGRAD: 1, OPT_ADAM: 2, OPT_FTRL: 2}.get(opt, 0)
        else:
            n_emb, n_w = state_arrays
            cfg.opt = OPT_NONE                     # each update call checks the arrays it needs
        mk = lambda *shape: torch.empty(shape, dtype=torch.float32, device=dev)
        self.acc_emb = mk(self.capacity, self.dim) if n_emb >= 1 else None
        self.acc2_emb = mk(self.capacity, self.dim) if n_emb >= 2 else None
        self.acc_w = mk(self.capacity) if n_w >= 1 else None
        self.acc2_w = mk(self.capacity) if n_w >= 2 else None
        self.row_keys = torch.empty((self.capacity,), dtype=torch.int64, device=dev)
        self.slots = torch.empty((sb.value,), dtype=torch.uint8, device=dev)
        self.workspace = torch.empty((wb.value,), dtype=torch.uint8, device=dev)
        cfg.emb, cfg.w, cfg.acc_emb, cfg.acc_w = _ptr(self.emb), _ptr(self.w), _ptr(self.acc_emb), _ptr(self.acc_w)
        cfg.row_keys, cfg.slots, cfg.slots_bytes = _ptr(self.row_keys), _ptr(self.slots), sb.value
        cfg.workspace, cfg.workspace_bytes = _ptr(self.workspace), wb.value
        cfg.acc2_emb, cfg.acc2_w = _ptr(self.acc2_emb), _ptr(self.acc2_w)
        self.cfg = cfg
        torch.cuda.synchronize()
        h = vp()
        _check(_lib.des_table_create(C.byref(cfg), C.byref(h)), "des_table_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            _lib.des_table_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- table ------------------------------------------------------------------------------
    def insert(self, keys: torch.Tensor, values: Optional[torch.Tensor] = None, rows_out: Optional[torch.Tensor] = None):
        _check(_lib.des_table_insert(self._h, _ptr(keys), keys.numel(), _ptr(values), _ptr(rows_out), _stream()),
               "des_table_insert")
        return rows_out

    def find(self, keys: torch.Tensor, miss: int = MISS_ZERO, rows_out: Optional[torch.Tensor] = None):
        if rows_out is None:
            rows_out = torch.empty(keys.numel(), dtype=torch.int32, device=keys.device)
        _check(_lib.des_table_find(self._h, _ptr(keys), keys.numel(), miss, _ptr(rows_out), _stream()), "des_table_find")
        return rows_out

    def migrate_into(self, dst: "Table", keep: Optional[torch.Tensor] = None, src_aux: Optional[torch.Tensor] = None,
                     dst_aux: Optional[torch.Tensor] = None) -> int:
        """Move the rows with keep[r] != 0 (uint8 device tensor; None = all) into the empty table `dst`
        (des_table_migrate); returns dst's row count."""
        n = i64(0)
        _check(_lib.des_table_migrate(self._h, _ptr(keep), dst._h, _ptr(src_aux), _ptr(dst_aux), C.byref(n), _stream()),
               "des_table_migrate")
        return int(n.value)

    def compact(self, keep: Optional[torch.Tensor], staging: torch.Tensor, aux: Optional[torch.Tensor] = None) -> int:
        """Drop the rows with keep[r] == 0 in place (des_table_compact); returns the new row count."""
        n = i64(0)
        _check(_lib.des_table_compact(self._h, _ptr(keep), _ptr(aux), _ptr(staging), staging.numel() * staging.element_size(),
                                      C.byref(n), _stream()), "des_table_compact")
        return int(n.value)

    def validate(self, batch: "Batch", rows: Optional[torch.Tensor] = None) -> int:
        """-1 if the batch (and rows) keep the contract the kernels rely on, else the index of the first
        offending offset, or B*F+1+e for rows[e] (des_batch_validate; synchronises)."""
        bad = i64(-1)
        code = _lib.des_batch_validate(self._h, C.byref(batch.desc), _ptr(rows), C.byref(bad), _stream())
        if code not in (OK, ERR_INVALID_ARG) or (code == ERR_INVALID_ARG and bad.value < 0):
            raise DesError(code, "des_batch_validate")
        return int(bad.value)

    def size(self) -> int:
        n = i64(0)
        _check(_lib.des_table_size(self._h, C.byref(n)), "des_table_size")
        return int(n.value)

    def status(self) -> int:
        return int(_lib.des_table_status(self._h))

    def clear_status(self):
        _check(_lib.des_table_clear_status(self._h), "des_table_clear_status")

    def export_keys(self, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """IDs of the rows in use, in row order (int64 tensor holding the uint64 bit patterns)."""
        if out is None:
            out = torch.empty(self.size(), dtype=torch.int64, device=self.emb.device)
        _check(_lib.des_table_export_keys(self._h, _ptr(out), out.numel(), _stream()), "des_table_export_keys")
        return out

    # ---- forward ----------------------------------------------------------------------------
    def partial_forward_lr(self, batch: Batch, rows, P_lr):
        _check(_lib.des_partial_forward_lr(self._h, C.byref(batch.desc), _ptr(rows), _ptr(P_lr), _stream()),
               "des_partial_forward_lr")

    def partial_forward_fm(self, batch: Batch, rows, P_sum, P_sq):
        _check(_lib.des_partial_forward_fm(self._h, C.byref(batch.desc), _ptr(rows), _ptr(P_sum), _ptr(P_sq), _stream()),
               "des_partial_forward_fm")

    def partial_forward_pool(self, batch: Batch, rows, P_pool, dense_k: bool):
        _check(_lib.des_partial_forward_pool(self._h, C.byref(batch.desc), _ptr(rows), _ptr(P_pool), int(dense_k),
                                             _stream()), "des_partial_forward_pool")

    def partial_forward(self, batch: Batch, rows, P_lr=None, P_sum=None, P_sq=None, pool=None):
        _check(_lib.des_partial_forward(self._h, C.byref(batch.desc), _ptr(rows), _ptr(P_lr), _ptr(P_sum), _ptr(P_sq),
                                        _ptr(pool), _stream()), "des_partial_forward")

    # ---- backward ---------------------------------------------------------------------------
    def _io(self, g_lr, g_fm, A_sum, g_pool, dbg):
        io = BackwardIO(_ptr(g_lr), _ptr(g_fm), _ptr(A_sum), _ptr(g_pool), None, None, None, None, None)
        if dbg:
            io.uniq_rows_out, io.uniq_keys_out = _ptr(dbg.get("uniq_rows")), _ptr(dbg.get("uniq_keys"))
            io.counts_out, io.merged_out, io.n_uniq_out = _ptr(dbg.get("counts")), _ptr(dbg.get("merged")), _ptr(dbg.get("n_uniq"))
        return io

    def backward_update_sgd(self, batch, rows, lr, g_lr=None, g_fm=None, A_sum=None, g_pool=None, dbg=None):
        io = self._io(g_lr, g_fm, A_sum, g_pool, dbg)
        _check(_lib.des_backward_update_sgd(self._h, C.byref(batch.desc), _ptr(rows), C.byref(io), lr, _stream()),
               "des_backward_update_sgd")

    def backward_update_adagrad(self, batch, rows, lr, eps, g_lr=None, g_fm=None, A_sum=None, g_pool=None, dbg=None):
        io = self._io(g_lr, g_fm, A_sum, g_pool, dbg)
        _check(_lib.des_backward_update_adagrad(self._h, C.byref(batch.desc), _ptr(rows), C.byref(io), lr, eps,
                                                _stream()), "des_backward_update_adagrad")

    def backward_update(self, batch, rows, optimizer: Optimizer, g_lr=None, g_fm=None, A_sum=None, g_pool=None, dbg=None):
        io = self._io(g_lr, g_fm, A_sum, g_pool, dbg)
        _check(_lib.des_backward_update(self._h, C.byref(batch.desc), _ptr(rows), C.byref(io), C.byref(optimizer),
                                        _stream()), "des_backward_update")

    def backward_prepare(self, batch, rows):
        """Row-sorting half of the next backward call for this batch, on the current stream."""
        _check(_lib.des_backward_prepare(self._h, C.byref(batch.desc), _ptr(rows), _stream()), "des_backward_prepare")

    def backward_merge(self, batch, rows, g_lr=None, g_fm=None, A_sum=None, g_pool=None, dbg=None):
        io = self._io(g_lr, g_fm, A_sum, g_pool, dbg)
        _check(_lib.des_backward_merge(self._h, C.byref(batch.desc), _ptr(rows), C.byref(io), _stream()),
               "des_backward_merge")

    def debug_buffers(self, nnz: int):
        dev = self.emb.device
        return {"uniq_rows": torch.empty(nnz, dtype=torch.int32, device=dev),
                "uniq_keys": torch.empty(nnz, dtype=torch.int64, device=dev),
                "counts": torch.empty(nnz, dtype=torch.int32, device=dev),
                "merged": torch.empty((nnz, self.dim + 1), dtype=torch.float32, device=dev),
                "n_uniq": torch.zeros(1, dtype=torch.int64, device=dev)}


def migrate_bytes(n_rows: int) -> int:
    n = C.c_size_t(0)
    _check(_lib.des_table_migrate_bytes(n_rows, C.byref(n)), "des_table_migrate_bytes")
    return int(n.value)


def mark_seen(rows: torch.Tensor, stamp: int, last_seen: torch.Tensor):
    """last_seen[rows[e]] = stamp for the entries with a row (last_seen: int32 tensor holding uint32 stamps)."""
    _check(_lib.des_table_mark_seen(_ptr(rows), rows.numel(), stamp, _ptr(last_seen), _stream()), "des_table_mark_seen")


def select_recent(last_seen: torch.Tensor, n_rows: int, min_stamp: int, keep: Optional[torch.Tensor] = None):
    if keep is None:
        keep = torch.empty(n_rows, dtype=torch.uint8, device=last_seen.device)
    _check(_lib.des_table_select_recent(_ptr(last_seen), n_rows, min_stamp, _ptr(keep), _stream()),
           "des_table_select_recent")
    return keep


def aggregate_partials(P: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    K = P.shape[0]
    n = P.numel() // K
    if out is None:
        out = torch.empty(P.shape[1:], dtype=torch.float32, device=P.device)
    _check(_lib.des_aggregate_partials(_ptr(P), K, n, _ptr(out), _stream()), "des_aggregate_partials")
    return out


def aggregate_forward(P_lr, P_sum, P_sq, A_lr=None, A_sum=None, A_sq=None, fm2=None):
    """All aggregations of one forward pass and fm2 in one launch (des_aggregate_forward)."""
    ref = P_sum if P_sum is not None else P_lr
    K, B = ref.shape[0], ref.shape[1]
    D = P_sum.shape[2] if P_sum is not None else 4
    _check(_lib.des_aggregate_forward(_ptr(P_lr), _ptr(P_sum), _ptr(P_sq), K, B, D, _ptr(A_lr), _ptr(A_sum), _ptr(A_sq),
                                      _ptr(fm2), _stream()), "des_aggregate_forward")


def fm_finalize(A_sum: torch.Tensor, A_sq: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    B, D = A_sum.shape
    if out is None:
        out = torch.empty(B, dtype=torch.float32, device=A_sum.device)
    _check(_lib.des_fm_finalize(_ptr(A_sum), _ptr(A_sq), B, D, _ptr(out), _stream()), "des_fm_finalize")
    return out


def dnn_partial_forward(pool: torch.Tensor, W: torch.Tensor, K: int,
                        out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y_partial[K,B,H] of the first fully-connected layer; pool [B,F,D], W [F*D,H], fp32 on the device."""
    B, F, D = pool.shape
    H = W.shape[1]
    if W.shape[0] != F * D or not (pool.is_contiguous() and W.is_contiguous()):
        raise ValueError("W must be [F*D, H]; both operands contiguous")
    if out is None:
        out = torch.empty((K, B, H), dtype=torch.float32, device=pool.device)
    _check(_lib.des_dnn_partial_forward(_ptr(pool), _ptr(W), B, F, D, H, K, _ptr(out), _stream()),
           "des_dnn_partial_forward")
    return out


def dnn_backward_bytes(B: int, F: int, D: int, H: int) -> int:
    n = C.c_size_t(0)
    _check(_lib.des_dnn_backward_bytes(B, F, D, H, C.byref(n)), "des_dnn_backward_bytes")
    return int(n.value)


def dnn_backward(pool: torch.Tensor, W: torch.Tensor, dY: torch.Tensor, g_pool: Optional[torch.Tensor],
                 dW: Optional[torch.Tensor], workspace: Optional[torch.Tensor] = None):
    """g_pool[B,F,D] = dY W^T and dW[F*D,H] = V dY into the given tensors (either may be None)."""
    B, F, D = pool.shape
    H = W.shape[1]
    if W.shape[0] != F * D or tuple(dY.shape) != (B, H):
        raise ValueError("shape mismatch")
    for t in (pool, W, dY, g_pool, dW):
        if t is not None and not t.is_contiguous():
            raise ValueError("operands must be contiguous")
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.des_dnn_backward(_ptr(pool), _ptr(W), _ptr(dY), B, F, D, H, _ptr(g_pool), _ptr(dW),
                                 _ptr(workspace), nbytes, _stream()), "des_dnn_backward")
    return g_pool, dW


def cross_partial(xl: torch.Tensor, w: torch.Tensor, K: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Per-shard scalars P[K,B] of a DCN cross layer: xl [B,F,D], w [F*D]; shard of field f is f mod K."""
    B, F, D = xl.shape
    if tuple(w.shape) != (F * D,) or not (xl.is_contiguous() and w.is_contiguous()):
        raise ValueError("xl must be contiguous [B,F,D] and w [F*D]")
    if out is None:
        out = torch.empty((K, B), dtype=torch.float32, device=xl.device)
    _check(_lib.des_cross_partial(_ptr(xl), _ptr(w), B, F, D, K, _ptr(out), _stream()), "des_cross_partial")
    return out


def cross_apply(x0: torch.Tensor, xl: torch.Tensor, s: torch.Tensor, bias: torch.Tensor,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """y = x0 * s[:,None] + bias + xl over rows of length d = x0.numel() / B."""
    B = x0.shape[0]
    d = bias.numel()
    if x0.numel() != B * d or xl.shape != x0.shape or s.numel() != B:
        raise ValueError("shape mismatch")
    if out is None:
        out = torch.empty_like(x0)
    for t in (x0, xl, s, bias, out):
        if not t.is_contiguous():
            raise ValueError("operands must be contiguous")
    _check(_lib.des_cross_apply(_ptr(x0), _ptr(xl), _ptr(s), _ptr(bias), B, d, _ptr(out), _stream()), "des_cross_apply")
    return out


def cross_backward_bytes(B: int, d: int) -> int:
    n = C.c_size_t(0)
    _check(_lib.des_cross_backward_bytes(B, d, C.byref(n)), "des_cross_backward_bytes")
    return int(n.value)


def cross_partial_backward(xl: torch.Tensor, w: torch.Tensor, g_s: torch.Tensor, g_xl: Optional[torch.Tensor],
                           dw: torch.Tensor, workspace: torch.Tensor):
    """g_xl = g_s[:,None] * w and dw = sum_b g_s[b] xl[b] for a gradient g_s of the aggregated scalar."""
    B = xl.shape[0]
    d = w.numel()
    if xl.numel() != B * d or g_s.numel() != B or dw.numel() != d or (g_xl is not None and g_xl.numel() != B * d):
        raise ValueError("shape mismatch")
    _check(_lib.des_cross_partial_backward(_ptr(xl), _ptr(w), _ptr(g_s), B, d, _ptr(g_xl), _ptr(dw), _ptr(workspace),
                                           _nbytes(workspace), _stream()), "des_cross_partial_backward")


def cross_backward(x0: torch.Tensor, xl: torch.Tensor, w: torch.Tensor, s: torch.Tensor, g_y: torch.Tensor,
                   g_xl: Optional[torch.Tensor], g_x0: torch.Tensor, accumulate_g_x0: bool, dw: torch.Tensor,
                   db: torch.Tensor, workspace: torch.Tensor):
    """Gradients of one cross layer into g_xl, g_x0 (added to when `accumulate_g_x0`), dw, db.  g_xl None: the
    layer's input is x0 itself and its gradient is added into g_x0 too."""
    B = x0.shape[0]
    d = w.numel()
    for t in (x0, xl, g_y, g_xl, g_x0):
        if t is None:
            continue
        if t.numel() != B * d or not t.is_contiguous():
            raise ValueError("row arrays must be contiguous with B*d elements")
    if s.numel() != B or dw.numel() != d or db.numel() != d:
        raise ValueError("shape mismatch")
    _check(_lib.des_cross_backward(_ptr(x0), _ptr(xl), _ptr(w), _ptr(s), _ptr(g_y), B, d, _ptr(g_xl), _ptr(g_x0),
                                   int(accumulate_g_x0), _ptr(dw), _ptr(db), _ptr(workspace), _nbytes(workspace),
                                   _stream()), "des_cross_backward")


def cross_net_bytes(B: int, d: int, n_layers: int) -> int:
    n = C.c_size_t(0)
    _check(_lib.des_cross_net_bytes(B, d, n_layers, C.byref(n)), "des_cross_net_bytes")
    return int(n.value)


def cross_net_partial(x0: torch.Tensor, U: torch.Tensor, K: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """P[K,B,m]: per-shard dot products of x0 [B,F,D] with the m rows of U [m, F*D]."""
    B, F, D = x0.shape
    m = U.shape[0]
    if U.shape[1] != F * D or not (x0.is_contiguous() and U.is_contiguous()):
        raise ValueError("x0 must be contiguous [B,F,D] and U contiguous [m,F*D]")
    if out is None:
        out = torch.empty((K, B, m), dtype=torch.float32, device=x0.device)
    _check(_lib.des_cross_net_partial(_ptr(x0), _ptr(U), B, F, D, m, K, _ptr(out), _stream()), "des_cross_net_partial")
    return out


def cross_net_forward(t: torch.Tensor, U: torch.Tensor, bias: Optional[torch.Tensor], gamma: torch.Tensor,
                      c: torch.Tensor, workspace: torch.Tensor):
    """gamma[B,m] and the logit term c[B] of the whole cross network from the aggregated dot products t[B,m]."""
    B, m = t.shape
    _check(_lib.des_cross_net_forward(_ptr(t), _ptr(U), _ptr(bias), B, U.shape[1], m - 1, _ptr(gamma), _ptr(c),
                                      _ptr(workspace), _nbytes(workspace), _stream()), "des_cross_net_forward")


def cross_net_backward(x0: torch.Tensor, U: torch.Tensor, bias: Optional[torch.Tensor], t: torch.Tensor,
                       gamma: torch.Tensor, g: torch.Tensor, g_x0: torch.Tensor, accumulate_g_x0: bool,
                       dU: torch.Tensor, dbias: Optional[torch.Tensor], workspace: torch.Tensor):
    """Backward of the whole cross network for the gradient g[B] of its logit term."""
    B = x0.shape[0]
    m, d = U.shape
    if x0.numel() != B * d or g_x0.numel() != B * d or tuple(t.shape) != (B, m) or tuple(gamma.shape) != (B, m):
        raise ValueError("shape mismatch")
    _check(_lib.des_cross_net_backward(_ptr(x0), _ptr(U), _ptr(bias), _ptr(t), _ptr(gamma), _ptr(g), B, d, m - 1,
                                       _ptr(g_x0), int(accumulate_g_x0), _ptr(dU), _ptr(dbias), _ptr(workspace),
                                       _nbytes(workspace), _stream()), "des_cross_net_backward")


def aggregate_bias_act(P: torch.Tensor, bias: Optional[torch.Tensor], relu: bool,
                       out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out[r,h] = act(sum_s P[s,r,h] + bias[h]); P is [K, rows, H]."""
    K, rows, H = P.shape
    if out is None:
        out = torch.empty((rows, H), dtype=torch.float32, device=P.device)
    _check(_lib.des_aggregate_bias_act(_ptr(P), K, rows, H, _ptr(bias), int(relu), _ptr(out), _stream()),
           "des_aggregate_bias_act")
    return out


def dense_workspace_bytes(H_max: int) -> int:
    n = C.c_size_t(0)
    _check(_lib.des_dense_workspace_bytes(H_max, C.byref(n)), "des_dense_workspace_bytes")
    return int(n.value)


def _nbytes(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def bias_act_backward(A: torch.Tensor, dA: torch.Tensor, relu: bool, dZ: torch.Tensor, dbias: torch.Tensor,
                      workspace: torch.Tensor):
    rows, H = A.shape
    _check(_lib.des_bias_act_backward(_ptr(A), _ptr(dA), rows, H, int(relu), _ptr(dZ), _ptr(dbias), _ptr(workspace),
                                      _nbytes(workspace), _stream()), "des_bias_act_backward")
    return dZ, dbias


def bias_act_backward_static(A: torch.Tensor, dA: torch.Tensor, relu: bool, dZ: torch.Tensor, dbias: torch.Tensor):
    """des_bias_act_backward with the library's own scratch array (allocates nothing; H <= 4096)."""
    rows, H = A.shape
    _check(_lib.des_bias_act_backward_static(_ptr(A), _ptr(dA), rows, H, int(relu), _ptr(dZ), _ptr(dbias), _stream()),
           "des_bias_act_backward_static")
    return dZ, dbias


def head(labels: torch.Tensor, g_logit: torch.Tensor, workspace: torch.Tensor, A_lr=None, fm2=None, a=None,
         w_out=None, b0=None, logit=None, p=None, loss=None, da=None, dw_out=None, db0=None):
    """Output unit + mean log-loss + gradients (see des_head); every tensor is a device fp32 tensor."""
    B = labels.shape[0]
    H = 0 if a is None else a.shape[1]
    _check(_lib.des_head(_ptr(A_lr), _ptr(fm2), _ptr(a), _ptr(w_out), _ptr(b0), _ptr(labels), B, H, _ptr(logit),
                         _ptr(p), _ptr(loss), _ptr(g_logit), _ptr(da), _ptr(dw_out), _ptr(db0), _ptr(workspace),
                         _nbytes(workspace), _stream()), "des_head")


def dense_update(theta: torch.Tensor, grad: torch.Tensor, optimizer: Optimizer, s1=None, s2=None):
    _check(_lib.des_dense_update(_ptr(theta), _ptr(grad), _ptr(s1), _ptr(s2), theta.numel(), C.byref(optimizer),
                                 _stream()), "des_dense_update")


def ceiling_gather(emb: torch.Tensor, rows: torch.Tensor, sink: Optional[torch.Tensor] = None,
                   w: Optional[torch.Tensor] = None) -> torch.Tensor:
    """des_ceiling_gather on the rows of a table's emb array, optionally with the LR weight fetch (measurement aid)."""
    if sink is None:
        n = C.c_size_t(0)
        _check(_lib.des_ceiling_gather_bytes(C.byref(n)), "des_ceiling_gather_bytes")
        sink = torch.empty(n.value // 4, dtype=torch.float32, device=emb.device)
    _check(_lib.des_ceiling_gather(_ptr(emb), emb.shape[1], emb.shape[1], _ptr(w), 1, emb.shape[0], _ptr(rows),
                                   rows.numel(), _ptr(sink), _nbytes(sink), _stream()), "des_ceiling_gather")
    return sink


def ceiling_update(emb: torch.Tensor, acc: torch.Tensor, uniq_rows: torch.Tensor):
    """des_ceiling_update: read and write back the listed rows of both arrays (measurement aid)."""
    _check(_lib.des_ceiling_update(_ptr(emb), _ptr(acc), emb.shape[1], emb.shape[1], emb.shape[0], _ptr(uniq_rows),
                                   uniq_rows.numel(), _stream()), "des_ceiling_update")


def profile_enable(on: bool):
    _check(_lib.des_profile_enable(int(on)), "des_profile_enable")


def profile_read():
    buf = (KernelTime * 64)()
    n = i32(0)
    _check(_lib.des_profile_read(buf, 64, C.byref(n)), "des_profile_read")
    return {buf[i].name.decode(): (int(buf[i].launches), float(buf[i].total_ms)) for i in range(n.value)}
