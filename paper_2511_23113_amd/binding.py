"""ctypes binding of libdbsp's C ABI (include/dbsp.h): argument marshalling only.

Every step of the hot path runs inside the library; nothing here computes.  The library is
loaded from this package's directory; if it has not been built yet it is built once with
hipcc, and any failure to build or load raises -- there is no CPU fallback.
"""

from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

DBSP_OK, DBSP_EINVAL, DBSP_ESHAPE, DBSP_ENOMEM, DBSP_EHIP = 0, -1, -2, -3, -4
MODE_BALANCED, MODE_NAIVE, MODE_ROUNDS, MODE_REWARD = 0, 1, 2, 3
PLAN_HOST_ONLY = 1
PLAN_PAIR_ROWS = 2
PLAN_PAIR_AUTO = 4

ROW_PTR, KV_IDX, ITEMS, ITEM_SLOT, SPLIT_ROWS, PART_PTR, PART_ITEMS, PART_LOAD, BLOCKS_PER_HEAD, ROW_CNT, EMPTY_ROWS, TAIL_ITEMS = range(12)
_INT64_ARRAYS = (PART_LOAD, BLOCKS_PER_HEAD)

EXPORTS = (
    "plan_sparse_attn", "plan_sparse_attn_reuse", "sparse_attn_fwd", "sparse_attn_fwd_static", "imbalance_ratio", "dbsp_plan_get", "dbsp_plan_stats",
    "dbsp_plan_busy", "dbsp_plan_tail_takes", "dbsp_plan_pair_rows", "dbsp_plan_calibrate", "dbsp_plan_destroy", "dbsp_last_error",
    "dbsp_partition_heads", "dbsp_partition_blocks", "dbsp_ring_work", "dbsp_fit_cost_model", "dbsp_mfma_probe",
)


class DbspError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libdbsp error {code}: {msg}")
        self.code = code


class PlanOpts(C.Structure):
    _fields_ = [("num_partitions", C.c_int32), ("mode", C.c_int32), ("max_item_len", C.c_int32),
                ("item_overhead", C.c_int32), ("flags", C.c_int32), ("locality_groups", C.c_int32),
                ("partition_cost", C.c_void_p), ("max_batch", C.c_int32), ("dynamic_tail", C.c_int32), ("reward", C.c_double),
                ("head_dim", C.c_int32)]


_lib = None


def load_library(path: str | None = None):
    """Load libdbsp.so (building it first if it does not exist).  Raises if that fails."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or _build.LIB_PATH
    if not os.path.exists(path):
        _build.build()
    lib = C.CDLL(path)
    vp, i32, i64p = C.c_void_p, C.c_int32, C.POINTER(C.c_int64)
    lib.plan_sparse_attn.argtypes = [vp, i32, i32, i32, i32, C.POINTER(PlanOpts), C.POINTER(vp)]
    lib.plan_sparse_attn.restype = C.c_int
    lib.plan_sparse_attn_reuse.argtypes = [vp, vp, C.POINTER(PlanOpts), C.c_double, C.POINTER(vp), C.POINTER(C.c_int32), C.POINTER(C.c_double)]
    lib.plan_sparse_attn_reuse.restype = C.c_int
    i32, i64, f64 = C.c_int32, C.c_int64, C.c_double
    lib.dbsp_partition_heads.argtypes = [vp, i32, i32, i32, vp, f64, vp, vp, vp, vp, C.POINTER(f64), C.POINTER(f64), C.POINTER(f64), C.POINTER(i32)]
    lib.dbsp_partition_heads.restype = C.c_int
    lib.dbsp_partition_blocks.argtypes = [vp, i32, i32, i32, i32, f64, i32, i32, vp, vp, vp, vp, vp, vp, vp,
                                          C.POINTER(f64), C.POINTER(f64), C.POINTER(i64), C.POINTER(i64)]
    lib.dbsp_partition_blocks.restype = C.c_int
    lib.dbsp_ring_work.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, C.POINTER(f64)]
    lib.dbsp_ring_work.restype = C.c_int
    lib.dbsp_fit_cost_model.argtypes = [vp, vp, vp, i32, C.POINTER(f64), C.POINTER(f64), C.POINTER(f64), C.POINTER(f64)]
    lib.dbsp_fit_cost_model.restype = C.c_int
    lib.dbsp_mfma_probe.argtypes = [C.POINTER(f64), C.POINTER(f64), vp]
    lib.dbsp_mfma_probe.restype = C.c_int
    lib.dbsp_plan_calibrate.argtypes = [vp, vp, vp]
    lib.dbsp_plan_calibrate.restype = C.c_int
    lib.sparse_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, C.c_float, vp]
    lib.sparse_attn_fwd.restype = C.c_int
    lib.sparse_attn_fwd_static.argtypes = lib.sparse_attn_fwd.argtypes
    lib.sparse_attn_fwd_static.restype = C.c_int
    lib.imbalance_ratio.argtypes = [vp, i32, i32, C.POINTER(C.c_double)]
    lib.imbalance_ratio.restype = C.c_int
    lib.dbsp_plan_get.argtypes = [vp, i32, C.POINTER(vp), i64p]
    lib.dbsp_plan_get.restype = C.c_int
    lib.dbsp_plan_stats.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), i64p, i64p,
                                    C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_double)]
    lib.dbsp_plan_stats.restype = C.c_int
    lib.dbsp_plan_busy.argtypes = [vp, vp, vp, vp]
    lib.dbsp_plan_busy.restype = C.c_int
    lib.dbsp_plan_tail_takes.argtypes = [vp, vp, vp]
    lib.dbsp_plan_tail_takes.restype = C.c_int
    lib.dbsp_plan_pair_rows.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.dbsp_plan_pair_rows.restype = C.c_int
    lib.dbsp_plan_destroy.argtypes = [vp]
    lib.dbsp_plan_destroy.restype = None
    lib.dbsp_last_error.argtypes = []
    lib.dbsp_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc: int):
    if rc != DBSP_OK:
        raise DbspError(rc, load_library().dbsp_last_error().decode("utf-8", "replace"))


class Plan:
    """Owner of a dbsp_plan*; destroyed on close() or garbage collection."""

    def __init__(self, handle: int, H: int, nQ: int, nK: int, block: int, pair_rows: bool = False):
        self._h = C.c_void_p(handle)
        self.H, self.nQ, self.nK, self.block = H, nQ, nK, block      # nQ, nK: the mask's block grid
        self.pair_rows = pair_rows

    @property
    def handle(self):
        if not self._h:
            raise ValueError("plan already destroyed")
        return self._h

    def array(self, what: int) -> np.ndarray:
        """Copy of one plan array (see dbsp_plan_array in dbsp.h)."""
        data, count = C.c_void_p(), C.c_int64()
        _check(load_library().dbsp_plan_get(self.handle, what, C.byref(data), C.byref(count)))
        dt = np.int64 if what in _INT64_ARRAYS else np.int32
        if count.value == 0:
            return np.zeros(0, dtype=dt)
        ctype = C.c_int64 if dt is np.int64 else C.c_int32
        buf = C.cast(data, C.POINTER(ctype * count.value)).contents
        return np.frombuffer(buf, dtype=dt).copy()

    def stats(self, with_rho: bool = True) -> dict:
        """dbsp_plan_stats.  with_rho=False leaves out rho_naive / rho_balanced (the library works those
        out on request: each costs a placement pass unless it is the placement the plan uses)."""
        rn, rb, rp, pu = C.c_double(), C.c_double(), C.c_double(), C.c_double()
        nnz, ni = C.c_int64(), C.c_int64()
        P, L = C.c_int32(), C.c_int32()
        _check(load_library().dbsp_plan_stats(self.handle, C.byref(rn) if with_rho else None, C.byref(rb) if with_rho else None,
                                              C.byref(rp), C.byref(nnz), C.byref(ni), C.byref(P), C.byref(L), C.byref(pu)))
        out = dict(rho_plan=rp.value, nnz=nnz.value, n_items=ni.value, num_partitions=P.value, max_item_len=L.value, plan_usec=pu.value)
        if with_rho:
            out.update(rho_naive=rn.value, rho_balanced=rb.value)
        return out

    def busy(self, stream=None):
        """(busy ticks uint64 [P] at 100 MHz, hw ids uint32 [P]) of the last forward call; synchronises."""
        P = self.stats(with_rho=False)["num_partitions"]
        ticks = np.zeros(P, dtype=np.uint64)
        hw = np.zeros(P, dtype=np.uint32)
        _check(load_library().dbsp_plan_busy(self.handle, ticks.ctypes.data_as(C.c_void_p),
                                             hw.ctypes.data_as(C.c_void_p), _stream_ptr(stream)))
        return ticks, hw

    def tail_takes(self, stream=None):
        """How often each item of the shared queue was taken since the plan was made (uint32 [n_tail]); synchronises."""
        n = int(self.array(TAIL_ITEMS).shape[0])
        takes = np.zeros(n, dtype=np.uint32)
        _check(load_library().dbsp_plan_tail_takes(self.handle, takes.ctypes.data_as(C.c_void_p), _stream_ptr(stream)))
        return takes

    def calibrate(self, stream=None):
        """Relative time per block of every partition in the last forward call (int32 [P], mean about 1024):
        pass it as partition_cost to later plans with the same partition count.  Synchronises."""
        cost = np.zeros(self.stats(with_rho=False)["num_partitions"], dtype=np.int32)
        _check(load_library().dbsp_plan_calibrate(self.handle, cost.ctypes.data_as(C.c_void_p), _stream_ptr(stream)))
        return cost

    def close(self):
        if self._h:
            load_library().dbsp_plan_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def plan_sparse_attn(mask, block: int, num_partitions: int = 0, mode: int = MODE_BALANCED,
                     max_item_len: int = 0, item_overhead: int = 0, host_only: bool = False,
                     locality_groups: int = 0, partition_cost=None, max_batch: int = 0, dynamic_tail: int = 0,
                     reward: float = 0.0, pair_rows: bool = False, head_dim: int = 0) -> Plan:
    """mask: uint8 host array [H, nQ, nK]; returns a Plan (see dbsp.h: plan_sparse_attn)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if mask.ndim != 3:
        raise ValueError("mask must be [H, nQ, nK]")
    H, nQ, nK = mask.shape
    cost = np.ascontiguousarray(partition_cost, dtype=np.int32) if partition_cost is not None else None
    if cost is not None:
        if num_partitions == 0:
            num_partitions = int(cost.shape[0])      # one cost per partition: the array fixes their number
        if cost.ndim != 1 or cost.shape[0] != num_partitions:
            raise ValueError("partition_cost must hold one value per partition")
    if pair_rows not in (False, True, "auto"):
        raise ValueError('pair_rows is False, True or "auto"')
    flags = (PLAN_HOST_ONLY if host_only else 0) | (PLAN_PAIR_AUTO if pair_rows == "auto" else PLAN_PAIR_ROWS if pair_rows else 0)
    opts = PlanOpts(num_partitions, mode, max_item_len, item_overhead, flags, locality_groups,
                    cost.ctypes.data_as(C.c_void_p) if cost is not None else None, max_batch, dynamic_tail, float(reward),
                    head_dim)
    out = C.c_void_p()
    _check(load_library().plan_sparse_attn(mask.ctypes.data_as(C.c_void_p), H, nQ, nK, block, C.byref(opts), C.byref(out)))
    chosen = C.c_int32()
    _check(load_library().dbsp_plan_pair_rows(out, C.byref(chosen)))
    return Plan(out.value, H, nQ, nK, block, bool(chosen.value))


def plan_sparse_attn_reuse(previous: Plan, mask, reuse_threshold: float, num_partitions: int = 0, mode: int = MODE_BALANCED,
                           max_item_len: int = 0, item_overhead: int = 0, host_only: bool = False, locality_groups: int = 0,
                           partition_cost=None, max_batch: int = 0, dynamic_tail: int = 0):
    """Plan the next mask of a sequence, keeping `previous`'s placement while rho_s under it stays
    <= reuse_threshold (see dbsp.h: plan_sparse_attn_reuse).  Returns (Plan, reused, rho_under_previous)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if mask.shape != (previous.H, previous.nQ, previous.nK):
        raise ValueError("mask shape differs from the previous plan's")
    cost = np.ascontiguousarray(partition_cost, dtype=np.int32) if partition_cost is not None else None
    if cost is not None:
        if num_partitions == 0:
            num_partitions = int(cost.shape[0])      # one cost per partition: the array fixes their number
        if cost.ndim != 1 or cost.shape[0] != num_partitions:
            raise ValueError("partition_cost must hold one value per partition")
    flags = (PLAN_HOST_ONLY if host_only else 0) | (PLAN_PAIR_ROWS if previous.pair_rows else 0)   # pair rows are kept
    opts = PlanOpts(num_partitions, mode, max_item_len, item_overhead, flags, locality_groups,
                    cost.ctypes.data_as(C.c_void_p) if cost is not None else None, max_batch, dynamic_tail, 0.0)
    out, reused, rho = C.c_void_p(), C.c_int32(), C.c_double()
    _check(load_library().plan_sparse_attn_reuse(previous.handle, mask.ctypes.data_as(C.c_void_p), C.byref(opts),
                                                 float(reuse_threshold), C.byref(out), C.byref(reused), C.byref(rho)))
    return (Plan(out.value, previous.H, previous.nQ, previous.nK, previous.block, previous.pair_rows),
            bool(reused.value), rho.value)


def _stream_ptr(stream):
    if stream is None:
        import torch
        if torch.cuda.is_available():
            return C.c_void_p(torch.cuda.current_stream().cuda_stream)
        return C.c_void_p(0)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def sparse_attn_fwd(plan: Plan, q, k, v, o=None, lse=None, softmax_scale: float = 0.0, stream=None, want_lse: bool = True,
                    static_scratch: bool = False):
    """q [B,H,Nq,d], k/v [B,H,Nk,d]: contiguous bf16 torch tensors on the GPU.  Enqueues on
    `stream` (default: torch's current stream) and returns (o, lse) without synchronising.
    static_scratch=True calls sparse_attn_fwd_static (pass o and lse then: this wrapper allocates
    the ones it is not given)."""
    import torch
    for name, x in (("q", q), ("k", k), ("v", v)):
        if x.dtype != torch.bfloat16 or not x.is_cuda or not x.is_contiguous() or x.dim() != 4:
            raise ValueError(f"{name} must be a contiguous 4-d bf16 tensor on the GPU")
    B, H, Nq, d = q.shape
    Nk = k.shape[2]
    if k.shape != (B, H, Nk, d) or v.shape != k.shape or H != plan.H:
        raise ValueError("q/k/v shapes disagree with each other or with the plan")
    if o is None:
        o = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((B, H, Nq), dtype=torch.float32, device=q.device)
    lse_ptr = C.c_void_p(lse.data_ptr()) if lse is not None else C.c_void_p(0)
    entry = load_library().sparse_attn_fwd_static if static_scratch else load_library().sparse_attn_fwd
    _check(entry(plan.handle, C.c_void_p(q.data_ptr()), C.c_void_p(k.data_ptr()),
                 C.c_void_p(v.data_ptr()), C.c_void_p(o.data_ptr()), lse_ptr,
                 B, Nq, Nk, d, float(softmax_scale), _stream_ptr(stream)))
    return o, lse


def imbalance_ratio(work) -> float:
    """Eq. 1 of the paper on an integer matrix work[periods][partitions]."""
    w = np.ascontiguousarray(work, dtype=np.int64)
    if w.ndim == 1:
        w = w[None]
    rho = C.c_double()
    _check(load_library().imbalance_ratio(w.ctypes.data_as(C.c_void_p), w.shape[0], w.shape[1], C.byref(rho)))
    return rho.value


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _split(flat, ptr):
    return [flat[ptr[g]:ptr[g + 1]].tolist() for g in range(len(ptr) - 1)]


def partition_heads(blocks_per_head, x: int, capacity: int = 0, previous=None, reuse_threshold: float = 1.0) -> dict:
    """Head-level partitioning over x GPUs with plan reuse (see dbsp.h: dbsp_partition_heads)."""
    cnt = np.ascontiguousarray(blocks_per_head, dtype=np.int64)
    H = cnt.shape[0]
    prev = np.ascontiguousarray(previous, dtype=np.int32) if previous is not None else None
    if prev is not None and prev.shape != (H,):
        raise ValueError("previous plan must hold one GPU id per head")
    where, lst, ptr = np.empty(H, np.int32), np.empty(H, np.int32), np.empty(max(x, 0) + 1, np.int32)
    load = np.empty(max(x, 0), np.int64)
    rc_, rp_, r_, reused = C.c_double(), C.c_double(), C.c_double(), C.c_int32()
    _check(load_library().dbsp_partition_heads(_ptr(cnt), H, x, capacity, _ptr(prev), float(reuse_threshold), _ptr(where), _ptr(lst),
                                               _ptr(ptr), _ptr(load), C.byref(rc_), C.byref(rp_), C.byref(r_), C.byref(reused)))
    return dict(gpu_of_head=where.tolist(), lists=_split(lst, ptr), loads=load.tolist(), rho_contiguous=rc_.value,
                rho=r_.value, rho_previous=rp_.value, reused=bool(reused.value))


def partition_blocks(mask, y: int, reward: float = 0.0, capacity_q: int = 0, capacity_kv: int = 0) -> dict:
    """Block-level partitioning of a mask [H, nQ, nK] for a ring of y GPUs (see dbsp.h: dbsp_partition_blocks)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if mask.ndim != 3:
        raise ValueError("mask must be [H, nQ, nK]")
    H, nQ, nK = mask.shape
    yy = max(y, 0)
    gq, ql, qp = np.empty(nQ, np.int32), np.empty(nQ, np.int32), np.empty(yy + 1, np.int32)
    gk, kl, kp = np.empty(nK, np.int32), np.empty(nK, np.int32), np.empty(yy + 1, np.int32)
    work = np.empty((yy, yy), np.int64)
    rc_, r_, mq, mk = C.c_double(), C.c_double(), C.c_int64(), C.c_int64()
    _check(load_library().dbsp_partition_blocks(_ptr(mask), H, nQ, nK, y, float(reward), capacity_q, capacity_kv, _ptr(gq), _ptr(ql),
                                                _ptr(qp), _ptr(gk), _ptr(kl), _ptr(kp), _ptr(work), C.byref(rc_), C.byref(r_),
                                                C.byref(mq), C.byref(mk)))
    return dict(gpu_of_q=gq.tolist(), q_lists=_split(ql, qp), chunk_of_kv=gk.tolist(), kv_lists=_split(kl, kp),
                work=work.tolist(), rho=r_.value, rho_contiguous=rc_.value, moved_q=mq.value, moved_kv=mk.value)


def ring_work(mask, y: int, gpu_of_q=None, chunk_of_kv=None):
    """Eq. 3's work matrix [iteration][GPU] and its rho_s for given maps (None = contiguous layout)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    H, nQ, nK = mask.shape
    gq = np.ascontiguousarray(gpu_of_q, dtype=np.int32) if gpu_of_q is not None else None
    gk = np.ascontiguousarray(chunk_of_kv, dtype=np.int32) if chunk_of_kv is not None else None
    if (gq is not None and gq.shape != (nQ,)) or (gk is not None and gk.shape != (nK,)):
        raise ValueError("maps must hold one id per block")
    work = np.empty((max(y, 0), max(y, 0)), np.int64)
    rho = C.c_double()
    _check(load_library().dbsp_ring_work(_ptr(mask), H, nQ, nK, y, _ptr(gq), _ptr(gk), _ptr(work), C.byref(rho)))
    return work.tolist(), rho.value


def fit_cost_model(blocks, items, time):
    """Least-squares (a, c, t0, rms residual) of time = a*blocks + c*items + t0 (see dbsp.h: dbsp_fit_cost_model)."""
    b = np.ascontiguousarray(blocks, dtype=np.int64)
    i = np.ascontiguousarray(items, dtype=np.int64)
    t = np.ascontiguousarray(time, dtype=np.float64)
    if not (b.shape == i.shape == t.shape and b.ndim == 1):
        raise ValueError("blocks, items and time must be 1-D arrays of one length")
    a, c, t0, rms = C.c_double(), C.c_double(), C.c_double(), C.c_double()
    _check(load_library().dbsp_fit_cost_model(_ptr(b), _ptr(i), _ptr(t), b.shape[0], C.byref(a), C.byref(c), C.byref(t0), C.byref(rms)))
    return a.value, c.value, t0.value, rms.value


def mfma_probe(stream=None):
    """(sustained dense bf16 MFMA TFLOP/s, shader clock in GHz) measured on the current device (see dbsp.h: dbsp_mfma_probe)."""
    t, g = C.c_double(), C.c_double()
    _check(load_library().dbsp_mfma_probe(C.byref(t), C.byref(g), _stream_ptr(stream)))
    return t.value, g.value
