"""Thin ctypes binding of libshadowsync (argument marshalling only).

Function names mirror include/shadowsync.h.  PyTorch supplies device memory (the workspace
and batch tensors) and streams; every step of the path runs inside the library's HIP
kernels.  There is no fallback: if the built library is missing, load() raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libshadowsync.so")

SS_EASGD, SS_MA, SS_BMUF, SS_EASGD_LITERAL, SS_BMUF_NESTEROV = 0, 1, 2, 3, 4
SS_FP32, SS_BF16 = 0, 1
POOLING = {"sum": 0, "mean": 1}
MLP_PATHS = {"auto": 0, "layerwise": 1}
EMB_OPTIMIZERS = {"rowwise_adagrad": 0, "adam": 1}
ALGOS = {"easgd": SS_EASGD, "ma": SS_MA, "bmuf": SS_BMUF, "easgd_literal": SS_EASGD_LITERAL,
         "bmuf_nesterov": SS_BMUF_NESTEROV}

(DBG_POOLED, DBG_INTERACT, DBG_LOGITS, DBG_DENSE_GRAD, DBG_POOLED_GRAD, DBG_SORTED_ROWS,
 DBG_SORTED_POS, DBG_SEG_STARTS, DBG_NUM_UNIQUE, DBG_BAG_OF_POS) = range(10)
_DBG_DTYPE = {DBG_POOLED: np.float32, DBG_INTERACT: np.float32, DBG_LOGITS: np.float32,
              DBG_DENSE_GRAD: np.float32, DBG_POOLED_GRAD: np.float32,
              DBG_SORTED_ROWS: np.uint32, DBG_SORTED_POS: np.uint32,
              DBG_SEG_STARTS: np.uint32, DBG_NUM_UNIQUE: np.uint32, DBG_BAG_OF_POS: np.int32}
DBG_Z0, DBG_POOLED_PARTIALS, DBG_SORTED_BAG, DBG_HIDDEN_ACT = 10, 11, 12, 32
_DBG_DTYPE[DBG_SORTED_BAG] = np.int32

(K_NONE, K_GATHER, K_SORT, K_ROW_UPDATE_CHUNK, K_SYNC, K_MLP, K_INTERACT_FWD, K_INTERACT_BWD,
 K_ROW_UPDATE, K_MLP_FWD, K_MLP_DGRAD, K_MLP_WGRAD) = range(12)

EXPORTS = [
    "ss_workspace_bytes", "ss_init", "ss_destroy", "ss_last_error", "ss_init_tables_hash",
    "ss_write_rows", "ss_write_adagrad", "ss_init_dense", "ss_num_params", "ss_train_step", "ss_eval_step",
    "ss_shadow_sync", "ss_easgd_exchange", "ss_sync_round", "ss_shadow_start", "ss_shadow_stop", "ss_read_dense",
    "ss_write_dense", "ss_read_rows", "ss_read_debug", "ss_get_counters", "ss_profile_arm",
    "ss_profile_sample", "ss_profile_sample_class", "ss_profile_read", "ss_shadow_pace", "ss_metrics_read",
    "ss_metrics_reset", "ss_eval_step_static", "ss_write_adam_state", "ss_read_adam_state",
    "ss_plan_placement",
]


class ss_config(C.Structure):
    _fields_ = [("num_tables", C.c_int32), ("rows", C.POINTER(C.c_int64)),
                ("emb_dim", C.c_int32), ("num_dense", C.c_int32),
                ("n_bot", C.c_int32), ("bot_dims", C.POINTER(C.c_int32)),
                ("n_top", C.c_int32), ("top_dims", C.POINTER(C.c_int32)),
                ("num_replicas", C.c_int32), ("max_batch", C.c_int32),
                ("max_ids", C.c_int64), ("num_worker_slots", C.c_int32),
                ("mlp_prec", C.c_int32), ("lr_dense", C.c_float), ("lr_emb", C.c_float),
                ("adagrad_eps", C.c_float), ("seed", C.c_uint64), ("pooling", C.c_int32),
                ("mlp_path", C.c_int32), ("emb_optimizer", C.c_int32),
                ("adam_beta1", C.c_float), ("adam_beta2", C.c_float),
                ("emb_row_shards", C.c_int32), ("sort_digit_bits", C.c_int32)]


class ss_shard(C.Structure):
    _fields_ = [("table", C.c_int32), ("first_row", C.c_int64), ("rows", C.c_int64),
                ("cost", C.c_double), ("ps", C.c_int32)]


class ss_batch(C.Structure):
    _fields_ = [("batch", C.c_int32), ("num_ids", C.c_int64), ("dense", C.c_void_p),
                ("labels", C.c_void_p), ("indices", C.c_void_p), ("offsets", C.c_void_p)]


_lib = None


def load() -> C.CDLL:
    """Open the built library; raise if it has not been built (no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2003_03477_amd.build` "
            "(the HIP library is the only implementation of this path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    lib.ss_workspace_bytes.restype = C.c_size_t
    lib.ss_workspace_bytes.argtypes = [C.POINTER(ss_config)]
    lib.ss_init.argtypes = [C.POINTER(ss_config), vp, C.c_size_t, C.POINTER(vp)]
    lib.ss_destroy.restype = None
    lib.ss_destroy.argtypes = [vp]
    lib.ss_last_error.restype = C.c_char_p
    lib.ss_last_error.argtypes = [vp]
    lib.ss_init_tables_hash.argtypes = [vp, vp]
    lib.ss_write_rows.argtypes = [vp, i32, i64, i64, vp]
    lib.ss_write_adagrad.argtypes = [vp, i32, i64, i64, vp]
    lib.ss_write_adam_state.argtypes = [vp, i32, i64, i64, vp, vp]
    lib.ss_read_adam_state.argtypes = [vp, i32, vp, i64, vp, vp]
    lib.ss_plan_placement.argtypes = [i32, vp, vp, i32, i64, vp, i32, vp, vp]
    lib.ss_init_dense.argtypes = [vp, vp]
    lib.ss_num_params.restype = i64
    lib.ss_num_params.argtypes = [vp]
    lib.ss_train_step.argtypes = [vp, i32, i32, C.POINTER(ss_batch), vp, vp]
    lib.ss_eval_step.argtypes = [vp, i32, i32, C.POINTER(ss_batch), vp, vp]
    lib.ss_eval_step_static.argtypes = [vp, i32, C.POINTER(ss_batch), vp, vp, vp]
    lib.ss_shadow_sync.argtypes = [vp, i32, f32, f32, f32, vp]
    lib.ss_easgd_exchange.argtypes = [vp, i32, i32, f32, vp]
    lib.ss_sync_round.argtypes = [i32, i32, i64, i64, vp, vp, vp, vp, f32, f32, f32, vp]
    lib.ss_shadow_start.argtypes = [vp, i32, f32, f32, f32, vp]
    lib.ss_shadow_stop.argtypes = [vp]
    lib.ss_shadow_pace.argtypes = [vp, i64]
    lib.ss_metrics_read.argtypes = [vp, i32, vp]
    lib.ss_metrics_reset.argtypes = [vp, i32]
    lib.ss_read_dense.argtypes = [vp, i32, vp, i64]
    lib.ss_write_dense.argtypes = [vp, i32, vp, i64]
    lib.ss_read_rows.argtypes = [vp, i32, vp, i64, vp, vp]
    lib.ss_read_debug.argtypes = [vp, i32, i32, vp, C.c_size_t, C.POINTER(C.c_size_t)]
    lib.ss_get_counters.argtypes = [vp, vp, vp, vp]
    lib.ss_profile_arm.argtypes = [vp, C.c_uint32]
    lib.ss_profile_sample.argtypes = [vp, i32]
    lib.ss_profile_sample_class.argtypes = [vp, i32, i32]
    lib.ss_profile_read.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(C.c_double)]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if fn.restype is C.c_int:
            fn.restype = C.c_int
    _lib = lib
    return lib


class ShadowSyncError(RuntimeError):
    pass


def _np_ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        return None
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


@dataclass
class DeviceBatch:
    """A batch resident in HBM (torch tensors keep the memory alive)."""
    dense: "object"
    labels: "object"
    indices: "object"
    offsets: "object"
    batch: int
    num_ids: int

    def struct(self) -> ss_batch:
        return ss_batch(self.batch, self.num_ids, self.dense.data_ptr(), self.labels.data_ptr(),
                        self.indices.data_ptr() if self.num_ids else None,
                        self.offsets.data_ptr())


def upload_batch(b, device="cuda:0") -> DeviceBatch:
    """Copy a synth.Batch (or a (dense, labels, indices, offsets) tuple) to the device."""
    import torch
    dense, labels, indices, offsets = b.as_tuple() if hasattr(b, "as_tuple") else b
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(device)
    n = int(offsets[-1])
    idx = indices if n else np.zeros(1, np.int32)
    return DeviceBatch(t(dense, np.float32), t(labels, np.float32), t(idx, np.int32),
                       t(offsets, np.int32), int(dense.shape[0]), n)


class ShadowSync:
    """Owner of one library context and of the torch tensor that backs its workspace."""

    def __init__(self, rows: Sequence[int], emb_dim: int, bot_dims: Sequence[int],
                 top_dims: Sequence[int], num_replicas: int, max_batch: int, max_ids: int,
                 num_worker_slots: int = 1, bf16: bool = False, lr_dense: float = 0.01,
                 lr_emb: float = 0.01, adagrad_eps: float = 1e-8, seed: int = 0,
                 device: str = "cuda:0", pooling: str = "sum", mlp_path: str = "auto",
                 emb_optimizer: str = "rowwise_adagrad", adam_betas=(0.9, 0.999),
                 emb_row_shards: int = 1, sort_digit_bits: int = 0):
        import torch
        self.lib = load()
        self.torch = torch
        self.device = torch.device(device)
        self._rows = (C.c_int64 * len(rows))(*rows)
        self._bot = (C.c_int32 * len(bot_dims))(*bot_dims)
        self._top = (C.c_int32 * len(top_dims))(*top_dims)
        self.cfg = ss_config(len(rows), self._rows, emb_dim, bot_dims[0], len(bot_dims),
                             self._bot, len(top_dims), self._top, num_replicas, max_batch,
                             max_ids, num_worker_slots, SS_BF16 if bf16 else SS_FP32,
                             lr_dense, lr_emb, adagrad_eps, seed, POOLING[pooling],
                             MLP_PATHS[mlp_path], EMB_OPTIMIZERS[emb_optimizer],
                             adam_betas[0], adam_betas[1], emb_row_shards, sort_digit_bits)
        self.rows, self.emb_dim, self.K = list(rows), emb_dim, num_replicas
        self.T = len(rows)
        self.ctx = C.c_void_p()
        nbytes = self.lib.ss_workspace_bytes(C.byref(self.cfg))
        if nbytes == 0:
            raise ShadowSyncError(self.lib.ss_last_error(None).decode())
        self.workspace_bytes = nbytes
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
            base = (self.workspace.data_ptr() + 255) // 256 * 256
            rc = self.lib.ss_init(C.byref(self.cfg), base, nbytes, C.byref(self.ctx))
        if rc != 0:
            raise ShadowSyncError(f"ss_init: {self.lib.ss_last_error(None).decode()}")
        self.P = int(self.lib.ss_num_params(self.ctx))
        self._loss = torch.zeros(max(num_worker_slots, 1), dtype=torch.float32,
                                 device=self.device)

    # ------------------------------------------------------------------ helpers
    def _check(self, rc: int, what: str):
        if rc != 0:
            raise ShadowSyncError(f"{what} failed ({rc}): "
                                  f"{self.lib.ss_last_error(self.ctx).decode()}")

    def close(self):
        if self.ctx:
            self.lib.ss_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ------------------------------------------------------------------ init
    def ss_init_tables_hash(self, stream=None):
        self._check(self.lib.ss_init_tables_hash(self.ctx, _stream_handle(stream)),
                    "ss_init_tables_hash")

    def ss_write_rows(self, table: int, first_row: int, values: np.ndarray):
        v = np.ascontiguousarray(values, dtype=np.float32)
        self._check(self.lib.ss_write_rows(self.ctx, table, first_row, v.shape[0], _np_ptr(v)),
                    "ss_write_rows")

    def ss_write_adagrad(self, table: int, first_row: int, values: np.ndarray):
        v = np.ascontiguousarray(values, dtype=np.float32)
        self._check(self.lib.ss_write_adagrad(self.ctx, table, first_row, v.shape[0], _np_ptr(v)),
                    "ss_write_adagrad")

    def ss_write_adam_state(self, table: int, first_row: int, m: np.ndarray, v: np.ndarray):
        m = np.ascontiguousarray(m, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        self._check(self.lib.ss_write_adam_state(self.ctx, table, first_row, m.shape[0], _np_ptr(m),
                                                 _np_ptr(v)), "ss_write_adam_state")

    def ss_read_adam_state(self, table: int, rows: np.ndarray):
        r = np.ascontiguousarray(rows, dtype=np.int64)
        m = np.empty((len(r), self.emb_dim), dtype=np.float32)
        v = np.empty((len(r), self.emb_dim), dtype=np.float32)
        self._check(self.lib.ss_read_adam_state(self.ctx, table, _np_ptr(r), len(r), _np_ptr(m),
                                                _np_ptr(v)), "ss_read_adam_state")
        return m, v

    def ss_init_dense(self, w0: np.ndarray):
        w = np.ascontiguousarray(w0, dtype=np.float32)
        assert w.shape == (self.P,)
        self._check(self.lib.ss_init_dense(self.ctx, _np_ptr(w)), "ss_init_dense")

    # ------------------------------------------------------------------ hot path
    def ss_train_step(self, replica: int, slot: int, batch: DeviceBatch, stream=None,
                      loss_out=None):
        """Enqueue one worker iteration; returns the 1-element device tensor that will hold
        the mean log-loss (before the update)."""
        out = loss_out if loss_out is not None else self._loss[slot:slot + 1]
        st = batch.struct()
        self._check(self.lib.ss_train_step(self.ctx, replica, slot, C.byref(st),
                                           _stream_handle(stream), out.data_ptr()),
                    "ss_train_step")
        return out

    def ss_eval_step(self, replica: int, slot: int, batch: DeviceBatch, stream=None,
                     loss_out=None):
        out = loss_out if loss_out is not None else self._loss[slot:slot + 1]
        st = batch.struct()
        self._check(self.lib.ss_eval_step(self.ctx, replica, slot, C.byref(st),
                                          _stream_handle(stream), out.data_ptr()),
                    "ss_eval_step")
        return out

    def ss_eval_step_static(self, replica: int, batch: DeviceBatch, loss_out, logits_out=None,
                            stream=None):
        """Forward pass in the library's static scratch array (no worker slot, no allocation):
        loss_out / logits_out are caller-owned device tensors (1 float / [batch] floats)."""
        st = batch.struct()
        self._check(self.lib.ss_eval_step_static(
            self.ctx, replica, C.byref(st), _stream_handle(stream), loss_out.data_ptr(),
            None if logits_out is None else logits_out.data_ptr()), "ss_eval_step_static")
        return loss_out

    def ss_shadow_sync(self, algo, alpha: float, eta: float = 1.0, momentum: float = 0.0,
                       stream=None):
        a = ALGOS[algo] if isinstance(algo, str) else int(algo)
        self._check(self.lib.ss_shadow_sync(self.ctx, a, alpha, eta, momentum,
                                            _stream_handle(stream)), "ss_shadow_sync")

    def ss_easgd_exchange(self, replica: int, alpha: float, stream=None, algo="easgd"):
        a = ALGOS[algo] if isinstance(algo, str) else int(algo)
        self._check(self.lib.ss_easgd_exchange(self.ctx, a, replica, alpha,
                                               _stream_handle(stream)), "ss_easgd_exchange")

    def ss_shadow_start(self, algo, alpha: float, eta: float = 1.0, momentum: float = 0.0,
                        stream=None):
        a = ALGOS[algo] if isinstance(algo, str) else int(algo)
        self._check(self.lib.ss_shadow_start(self.ctx, a, alpha, eta, momentum,
                                             _stream_handle(stream)), "ss_shadow_start")

    def ss_shadow_stop(self):
        self._check(self.lib.ss_shadow_stop(self.ctx), "ss_shadow_stop")

    def ss_shadow_pace(self, min_period_us: int):
        self._check(self.lib.ss_shadow_pace(self.ctx, int(min_period_us)), "ss_shadow_pace")

    def ss_metrics_read(self, which: int):
        """(examples, mean log-loss, click rate, NE) of the train (0) or eval (1) accumulator."""
        out = np.zeros(4, dtype=np.float64)
        self._check(self.lib.ss_metrics_read(self.ctx, which, _np_ptr(out)), "ss_metrics_read")
        return tuple(float(v) for v in out)

    def ss_metrics_reset(self, which: int):
        self._check(self.lib.ss_metrics_reset(self.ctx, which), "ss_metrics_reset")

    # ------------------------------------------------------------------ read-back
    def ss_read_dense(self, which: int) -> np.ndarray:
        out = np.empty(self.P, dtype=np.float32)
        self._check(self.lib.ss_read_dense(self.ctx, which, _np_ptr(out), self.P), "ss_read_dense")
        return out

    def ss_write_dense(self, which: int, values: np.ndarray):
        v = np.ascontiguousarray(values, dtype=np.float32)
        self._check(self.lib.ss_write_dense(self.ctx, which, _np_ptr(v), v.shape[0]),
                    "ss_write_dense")

    def ss_read_rows(self, table: int, rows: np.ndarray):
        r = np.ascontiguousarray(rows, dtype=np.int64)
        vals = np.empty((len(r), self.emb_dim), dtype=np.float32)
        acc = np.empty(len(r), dtype=np.float32)
        self._check(self.lib.ss_read_rows(self.ctx, table, _np_ptr(r), len(r), _np_ptr(vals),
                                          _np_ptr(acc)), "ss_read_rows")
        return vals, acc

    def ss_read_debug(self, slot: int, item: int) -> np.ndarray:
        size = C.c_size_t(0)
        self._check(self.lib.ss_read_debug(self.ctx, slot, item, None, 0, C.byref(size)),
                    "ss_read_debug")
        out = np.empty(size.value // 4, dtype=_DBG_DTYPE.get(item, np.float32))
        if size.value:
            self._check(self.lib.ss_read_debug(self.ctx, slot, item, _np_ptr(out), size.value,
                                               None), "ss_read_debug")
        return out

    def ss_get_counters(self):
        steps = np.zeros(self.K, dtype=np.uint64)
        rounds, examples = C.c_uint64(0), C.c_uint64(0)
        self._check(self.lib.ss_get_counters(self.ctx, _np_ptr(steps), C.byref(rounds),
                                             C.byref(examples)), "ss_get_counters")
        return steps, int(rounds.value), int(examples.value)

    def ss_profile_arm(self, *kernel_ids: int):
        mask = 0
        for k in kernel_ids:
            mask |= 1 << k
        self._check(self.lib.ss_profile_arm(self.ctx, mask), "ss_profile_arm")

    def ss_profile_sample(self, every: int):
        """Bracket only every `every`-th launch of each armed kernel class."""
        self._check(self.lib.ss_profile_sample(self.ctx, every), "ss_profile_sample")

    def ss_profile_sample_class(self, kernel_id: int, every: int):
        """The same for one kernel class."""
        self._check(self.lib.ss_profile_sample_class(self.ctx, kernel_id, every),
                    "ss_profile_sample_class")

    def ss_profile_read(self, kernel_id: int):
        n, ms = C.c_int64(0), C.c_double(0.0)
        self._check(self.lib.ss_profile_read(self.ctx, kernel_id, C.byref(n), C.byref(ms)),
                    "ss_profile_read")
        return int(n.value), float(ms.value)


def ss_sync_round(algo, K: int, P: int, stride: int, replicas, w_ps=None, w_global=None, v=None,
                  alpha: float = 0.1, eta: float = 1.0, momentum: float = 0.0, stream=None):
    """One shadow round on caller-owned torch tensors (float32, device)."""
    lib = load()
    a = ALGOS[algo] if isinstance(algo, str) else int(algo)
    ptr = lambda t: None if t is None else t.data_ptr()
    rc = lib.ss_sync_round(a, K, P, stride, ptr(replicas), ptr(w_ps), ptr(w_global), ptr(v),
                           alpha, eta, momentum, _stream_handle(stream))
    if rc != 0:
        raise ShadowSyncError(f"ss_sync_round failed ({rc})")


def ss_plan_placement(rows, cost, num_ps: int, max_rows_per_shard: int = 0):
    """Host-side placement plan: ([(table, first_row, rows, cost, ps)], cost per PS)."""
    lib = load()
    r = np.ascontiguousarray(rows, dtype=np.int64)
    c = np.ascontiguousarray(cost, dtype=np.float64)
    n = C.c_int32(0)
    load_out = np.zeros(num_ps, dtype=np.float64)
    lib.ss_plan_placement(len(r), _np_ptr(r), _np_ptr(c), num_ps, max_rows_per_shard, None, 0,
                          C.byref(n), None)
    buf = (ss_shard * max(n.value, 1))()
    rc = lib.ss_plan_placement(len(r), _np_ptr(r), _np_ptr(c), num_ps, max_rows_per_shard, buf,
                               n.value, C.byref(n), _np_ptr(load_out))
    if rc != 0:
        raise ShadowSyncError(f"ss_plan_placement failed ({rc})")
    return [(s.table, s.first_row, s.rows, s.cost, s.ps) for s in buf[:n.value]], load_out.tolist()


def from_workload(wl, rows=None, num_worker_slots: int = 1, max_ids: Optional[int] = None,
                  device="cuda:0", mlp_path: str = "auto", sort_digit_bits: int = 0) -> ShadowSync:
    """Context sized for a synth.Workload (rows may be overridden by a compacted problem)."""
    rows = list(rows if rows is not None else wl.rows)
    if max_ids is None:
        lam = wl.bag_lambda + 1
        max_ids = int(wl.batch * wl.num_tables * (lam + 6 * (lam ** 0.5) / (wl.batch ** 0.5)) + 4096)
    return ShadowSync(rows, wl.emb_dim, wl.bot_dims, wl.top_dims, wl.num_replicas, wl.batch,
                      max_ids, num_worker_slots, wl.bf16, wl.lr_dense, wl.lr_emb,
                      wl.adagrad_eps, wl.seed, device, wl.pooling, mlp_path,
                      getattr(wl, "emb_optimizer", "rowwise_adagrad"),
                      getattr(wl, "adam_betas", (0.9, 0.999)), getattr(wl, "emb_row_shards", 1),
                      sort_digit_bits)
