"""Thin ctypes binding of ``libmgg.so``: same names as the C ABI in ``include/mgg.h``.

Argument marshalling only -- every step of the path runs inside the library's HIP kernels.
PyTorch appears here solely as the owner of device memory and of the stream handle.  There
is no CPU fallback: if the library is missing the import of any entry point raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmgg.so")

OK, ERR_INVALID_ARG, ERR_BAD_GRAPH, ERR_UNSUPPORTED, ERR_ALLOC, ERR_HIP = range(6)
F32, BF16 = 0, 1
AGG_GCN_SYM, AGG_GIN_SUM = 0, 1
ACT_NONE, ACT_RELU, ACT_SOFTMAX = 0, 1, 2
_MODE = {"gcn": AGG_GCN_SYM, "gin": AGG_GIN_SUM}
_ACT = {"none": ACT_NONE, "relu": ACT_RELU, "softmax": ACT_SOFTMAX}
ORDER_AGG_FIRST, ORDER_UPDATE_FIRST, ORDER_AUTO = 0, 1, 2
_ORDER = {"agg_first": ORDER_AGG_FIRST, "update_first": ORDER_UPDATE_FIRST, "auto": ORDER_AUTO}
_STATUS_NAME = ["OK", "INVALID_ARG", "BAD_GRAPH", "UNSUPPORTED", "ALLOC", "HIP"]

EXPORTED_SYMBOLS = [
    "mgg_build_partition", "mgg_partition_info", "mgg_partition_export", "mgg_partition_destroy",
    "mgg_partition_reserve", "mgg_aggregate_scratch_bytes", "mgg_aggregate", "mgg_aggregate_static", "mgg_aggregate_to", "mgg_build_bags", "mgg_bag_sum", "mgg_update", "mgg_update_mlp", "mgg_layer_workspace_bytes", "mgg_layer_forward",
    "mgg_split_edge_balanced", "mgg_set_option", "mgg_get_option", "mgg_partition_set_option", "mgg_partition_get_option", "mgg_time_aggregate", "mgg_probe_gather",
    "mgg_model_evaluate", "mgg_tuner_create", "mgg_tuner_set_constraint", "mgg_tuner_next", "mgg_tuner_report", "mgg_tuner_result",
    "mgg_tuner_table", "mgg_tuner_destroy", "mgg_tune_aggregate",
    "mgg_last_error", "mgg_version",
]


class MggError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"MGG_ERR_{_STATUS_NAME[status] if 0 <= status < 6 else status}: {message}")
        self.status = status


class BuildOpts(C.Structure):
    _fields_ = [("ps", C.c_int32), ("dist", C.c_int32), ("short_max", C.c_int32), ("host_only", C.c_int32),
                ("wpb", C.c_int32), ("xcd_min_deg", C.c_int32), ("hot_row_bytes", C.c_int32), ("hot_rows", C.c_int32),
                ("hot_phases", C.c_int32), ("min_piece", C.c_int32), ("hot_min_count", C.c_int32), ("reserve_dim", C.c_int32)]


class PartitionInfo(C.Structure):
    _fields_ = [("num_nodes", C.c_int64), ("lb", C.c_int64), ("ub", C.c_int64), ("n_own", C.c_int64),
                ("nnz_local", C.c_int64), ("nnz_remote", C.c_int64), ("num_halo", C.c_int64),
                ("num_parts", C.c_int32), ("part_id", C.c_int32),
                ("ps", C.c_int32), ("dist", C.c_int32), ("short_max", C.c_int32), ("on_device", C.c_int32),
                ("xcd_min_deg", C.c_int32), ("wpb", C.c_int32),
                ("class_mode", C.c_int32),
                ("hot_rows", C.c_int32), ("n_phases", C.c_int32), ("min_piece", C.c_int32), ("hot_min_count", C.c_int32),
                ("n_groups_local", C.c_int64), ("n_groups_remote", C.c_int64),
                ("n_short_rows", C.c_int64), ("n_items", C.c_int64),
                ("n_split_rows", C.c_int64), ("n_split_items", C.c_int64),
                ("n_local_rows", C.c_int64), ("is_bags", C.c_int32), ("reserved_dim", C.c_int32)]


_ARRAY_FIELDS = ["local_row_ptr", "local_col", "remote_row_ptr", "remote_col", "halo_gid", "halo_peer_ptr",
                 "deg_own", "deg_halo", "grp_local_row", "grp_local_start", "grp_local_end",
                 "grp_remote_row", "grp_remote_start", "grp_remote_end", "short_rows",
                 "sched_local_col", "sched_remote_col",
                 "item_row", "item_lbeg", "item_lend", "item_rbeg", "item_rend", "item_slot",
                 "src_class_local", "src_class_halo"]


class PartitionArrays(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in _ARRAY_FIELDS]


class Knobs(C.Structure):
    _fields_ = [("ps", C.c_int32), ("dist", C.c_int32), ("wpb", C.c_int32)]


class Model(C.Structure):
    _fields_ = [("wpw", C.c_int64), ("smem_bytes", C.c_int64), ("num_waves", C.c_int64), ("num_blocks", C.c_int64),
                ("blocks_per_unit", C.c_double), ("feasible", C.c_int32)]


class LayerDesc(C.Structure):
    _fields_ = [("mode", C.c_int), ("eps", C.c_float), ("n_linear", C.c_int32), ("dims", C.c_int32 * 3),
                ("w_dtype", C.c_int), ("w", C.c_void_p * 2), ("bias", C.c_void_p * 2), ("act", C.c_int * 2),
                ("order", C.c_int)]


_lib = None


def lib():
    """Load libmgg.so (built in-tree by ``paper_2209_06800_amd.build``); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2209_06800_amd.build` "
                              "(there is no fallback path)")
        # torch first: it ships its own HIP runtime under the same soname, and the stream
        # handles and device pointers handed to the library must belong to that runtime
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.mgg_last_error.restype = C.c_char_p
        L.mgg_version.restype = C.c_char_p
        L.mgg_layer_workspace_bytes.restype = C.c_size_t
        L.mgg_partition_destroy.restype = None
        L.mgg_partition_destroy.argtypes = [C.c_void_p]
        L.mgg_build_partition.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                          C.c_void_p, C.POINTER(C.c_void_p)]
        L.mgg_partition_info.argtypes = [C.c_void_p, C.POINTER(PartitionInfo)]
        L.mgg_partition_export.argtypes = [C.c_void_p, C.POINTER(PartitionArrays)]
        L.mgg_aggregate.argtypes = [C.c_void_p, C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_int32,
                                    C.c_int64, C.c_void_p, C.c_int64, C.c_void_p]
        L.mgg_aggregate_static.argtypes = L.mgg_aggregate.argtypes
        L.mgg_partition_reserve.argtypes = [C.c_void_p, C.c_int32]
        L.mgg_aggregate_scratch_bytes.restype = C.c_size_t
        L.mgg_aggregate_scratch_bytes.argtypes = [C.c_void_p, C.c_int32]
        L.mgg_aggregate_to.argtypes = [C.c_void_p, C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_int32,
                                       C.c_int64, C.c_int, C.c_void_p, C.c_int64, C.c_void_p]
        L.mgg_build_bags.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p,
                                     C.POINTER(C.c_void_p)]
        L.mgg_bag_sum.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int, C.c_void_p,
                                  C.c_int64, C.c_void_p]
        L.mgg_update.argtypes = [C.c_int64, C.c_int, C.c_void_p, C.c_int64, C.c_int32, C.c_int, C.c_void_p,
                                 C.c_void_p, C.c_int32, C.c_int, C.c_int, C.c_void_p, C.c_int64, C.c_void_p]
        L.mgg_update_mlp.argtypes = [C.c_int64, C.c_int, C.c_void_p, C.c_int64, C.POINTER(C.c_int32), C.c_int, C.c_void_p,
                                     C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int64, C.c_int,
                                     C.c_void_p, C.c_int64, C.c_void_p]
        L.mgg_layer_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(LayerDesc)]
        L.mgg_layer_forward.argtypes = [C.c_void_p, C.POINTER(LayerDesc), C.c_int, C.c_void_p, C.c_void_p,
                                        C.c_int64, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_int64,
                                        C.c_void_p]
        L.mgg_split_edge_balanced.argtypes = [C.c_int64, C.c_void_p, C.c_int32, C.c_void_p]
        L.mgg_set_option.argtypes = [C.c_char_p, C.c_int32]
        L.mgg_get_option.argtypes = [C.c_char_p, C.POINTER(C.c_int32)]
        L.mgg_partition_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int32]
        L.mgg_partition_get_option.argtypes = [C.c_void_p, C.c_char_p, C.POINTER(C.c_int32)]
        L.mgg_time_aggregate.argtypes = [C.c_void_p, C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_void_p,
                                         C.c_int32, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                                         C.POINTER(C.c_float)]
        L.mgg_probe_gather.argtypes = [C.c_int64, C.c_int32, C.c_int64, C.c_int32, C.c_uint64, C.POINTER(C.c_double)]
        L.mgg_model_evaluate.argtypes = [C.c_int64, C.c_int64, Knobs, C.c_int32, C.c_int32, C.c_int64,
                                         C.POINTER(Model)]
        L.mgg_tuner_create.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
        L.mgg_tuner_set_constraint.argtypes = [C.c_void_p, C.c_int32, C.c_int64]
        L.mgg_tuner_next.argtypes = [C.c_void_p, C.POINTER(Knobs), C.POINTER(C.c_int32)]
        L.mgg_tuner_report.argtypes = [C.c_void_p, C.c_double]
        L.mgg_tuner_result.argtypes = [C.c_void_p, C.POINTER(Knobs), C.POINTER(C.c_double), C.POINTER(C.c_int32)]
        L.mgg_tuner_table.argtypes = [C.c_void_p, C.c_int32, C.POINTER(Knobs), C.POINTER(C.c_double),
                                      C.POINTER(C.c_int32)]
        L.mgg_tuner_destroy.restype = None
        L.mgg_tuner_destroy.argtypes = [C.c_void_p]
        L.mgg_tune_aggregate.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                         C.c_void_p, C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_int32,
                                         C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p,
                                         C.POINTER(Knobs), C.POINTER(C.c_double)]
        _lib = L
    return _lib


def _check(status: int):
    if status != OK:
        raise MggError(status, lib().mgg_last_error().decode())


def mgg_version() -> str:
    return lib().mgg_version().decode()


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# ------------------------------------------------------------------------------- torch glue
def _torch_dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _dev_ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("device tensor expected")
    return C.c_void_p(t.data_ptr())


def _ld(t) -> int:
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("row-major 2-D tensor with unit column stride expected")
    return int(t.stride(0)) if t.shape[0] > 1 else max(int(t.stride(0)), int(t.shape[1]))


def _stream(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


# ------------------------------------------------------------------------------- partition
class Partition:
    """Owner of an ``mgg_partition_t*``."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)
        self.info = PartitionInfo()
        _check(lib().mgg_partition_info(self._h, C.byref(self.info)))
        self._reserved = int(self.info.reserved_dim)

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("partition already destroyed")
        return self._h

    def destroy(self):
        if self._h is not None:
            lib().mgg_partition_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def reserve(self, dim: int):
        """mgg_partition_reserve: size the partition's scratch buffer for aggregations up to `dim` wide."""
        if dim > self._reserved:
            _check(lib().mgg_partition_reserve(self.handle, int(dim)))
            self._reserved = int(dim)

    def set_option(self, key: str, value: int):
        """A run-time switch of this partition's aggregations (mgg_partition_set_option)."""
        _check(lib().mgg_partition_set_option(self.handle, key.encode(), int(value)))

    def get_option(self, key: str) -> int:
        v = C.c_int32()
        _check(lib().mgg_partition_get_option(self.handle, key.encode(), C.byref(v)))
        return v.value

    def export(self) -> dict:
        """Copy every integer structure to numpy arrays (for bit-exact checks)."""
        i = self.info
        sizes = {
            "local_row_ptr": i.n_own + 1, "local_col": i.nnz_local, "remote_row_ptr": i.n_own + 1,
            "remote_col": i.nnz_remote, "halo_gid": i.num_halo, "halo_peer_ptr": i.num_parts + 1,
            "deg_own": i.n_own, "deg_halo": i.num_halo,
            "grp_local_row": i.n_groups_local, "grp_local_start": i.n_groups_local, "grp_local_end": i.n_groups_local,
            "grp_remote_row": i.n_groups_remote, "grp_remote_start": i.n_groups_remote,
            "grp_remote_end": i.n_groups_remote, "short_rows": i.n_short_rows,
            "sched_local_col": i.nnz_local, "sched_remote_col": i.nnz_remote,
            "item_row": i.n_items, "item_lbeg": i.n_items, "item_lend": i.n_items, "item_rbeg": i.n_items,
            "item_rend": i.n_items, "item_slot": i.n_items,
            "src_class_local": i.n_local_rows, "src_class_halo": i.num_halo,
        }
        out = {k: np.zeros(max(int(n), 0), dtype=np.int64 if k == "halo_peer_ptr" else np.int32)
               for k, n in sizes.items()}
        arrs = PartitionArrays(**{k: out[k].ctypes.data for k in _ARRAY_FIELDS})
        _check(lib().mgg_partition_export(self.handle, C.byref(arrs)))
        return out


def mgg_build_partition(row_ptr: np.ndarray, col_idx: np.ndarray, num_parts: int = 1, part_id: int = 0,
                        bounds: Optional[Sequence[int]] = None, *, ps: int = 0, dist: int = 0,
                        short_max: int = 0, host_only: bool = False, xcd_min_deg: int = 0, wpb: int = 0,
                        hot_row_bytes: int = 0, hot_rows: int = 0, hot_phases: int = 0, min_piece: int = 0,
                        hot_min_count: int = 0, reserve_dim: int = 0, num_nodes: Optional[int] = None) -> Partition:
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    n = row_ptr.size - 1 if num_nodes is None else num_nodes
    b = None if bounds is None else np.ascontiguousarray(bounds, dtype=np.int64)
    if b is not None and b.size != num_parts + 1:
        raise MggError(ERR_INVALID_ARG, "bounds must have num_parts + 1 entries")
    opts = BuildOpts(ps, dist, short_max, int(host_only), wpb, xcd_min_deg, hot_row_bytes, hot_rows, hot_phases,
                     min_piece, hot_min_count, reserve_dim)
    h = C.c_void_p()
    _check(lib().mgg_build_partition(n, _np_ptr(row_ptr), _np_ptr(col_idx) if col_idx.size else None,
                                     num_parts, part_id, _np_ptr(b), C.byref(opts), C.byref(h)))
    return Partition(h.value)


def mgg_build_bags(bag_ptr: np.ndarray, bag_idx: np.ndarray, table_rows: int, local_lo: int, local_hi: int, *,
                   host_only: bool = False, **knobs) -> Partition:
    """Partition for an embedding-bag sum: bags as owned rows, lookups split by the local slice of the table."""
    bag_ptr = np.ascontiguousarray(bag_ptr, dtype=np.int64)
    bag_idx = np.ascontiguousarray(bag_idx, dtype=np.int32)
    opts = BuildOpts()
    opts.host_only = int(host_only)
    for key, v in knobs.items():
        setattr(opts, key, v)
    h = C.c_void_p()
    _check(lib().mgg_build_bags(bag_ptr.size - 1, _np_ptr(bag_ptr), _np_ptr(bag_idx) if bag_idx.size else None, table_rows,
                                local_lo, local_hi, C.byref(opts), C.byref(h)))
    return Partition(h.value)


def mgg_bag_sum(part: Partition, table_local, table_halo=None, *, out=None, out_dtype=None, dim: Optional[int] = None, stream=None):
    """out[num_bags x dim] = sum of the looked-up rows of every bag."""
    import torch
    ref = table_local if table_local is not None else table_halo
    dim = int(ref.shape[1]) if dim is None else dim
    if out is None:
        out = torch.empty((int(part.info.n_own), dim), dtype=out_dtype or torch.float32, device=ref.device)
    _check_tables(part, table_local, table_halo, out, dim, bags=True)
    part.reserve(dim)
    _check(lib().mgg_bag_sum(part.handle, _torch_dtype_code(ref), _dev_ptr(table_local), _dev_ptr(table_halo), dim, _ld(ref),
                             _torch_dtype_code(out), _dev_ptr(out), _ld(out), _stream(stream)))
    return out


def mgg_split_edge_balanced(row_ptr: np.ndarray, num_parts: int) -> np.ndarray:
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    out = np.zeros(num_parts + 1, dtype=np.int64)
    _check(lib().mgg_split_edge_balanced(row_ptr.size - 1, _np_ptr(row_ptr), num_parts, _np_ptr(out)))
    return out


def mgg_set_option(key: str, value: int):
    _check(lib().mgg_set_option(key.encode(), int(value)))


def mgg_get_option(key: str) -> int:
    v = C.c_int32()
    _check(lib().mgg_get_option(key.encode(), C.byref(v)))
    return v.value


# ------------------------------------------------------------------------------- device calls
def _check_tables(part: Partition, x_local, x_halo, out, dim: int, bags: bool = False):
    """The C ABI takes bare pointers and one leading dimension for both tables; what it cannot see is
    checked here: both tables of one dtype, device and row stride, and every buffer long enough."""
    i = part.info
    if bool(i.is_bags) != bags:
        return                      # the wrong kind of partition for this call: the library says so
    n_local = int(i.n_local_rows) if bags else int(i.n_own)
    ref = x_local if x_local is not None else x_halo
    if ref is None:
        if n_local or int(i.num_halo):
            raise ValueError("no embedding table given")
        return
    if x_local is not None and x_halo is not None:
        if x_halo.dtype != x_local.dtype or x_halo.device != x_local.device:
            raise ValueError(f"x_halo is {x_halo.dtype} on {x_halo.device}, x_local is {x_local.dtype} on {x_local.device}")
        if int(x_halo.shape[0]) > 0 and int(x_local.shape[0]) > 0 and _ld(x_halo) != _ld(x_local):
            raise ValueError(f"x_halo has row stride {_ld(x_halo)}, x_local {_ld(x_local)}: the library takes one ld_x for both tables")
    for name, t, rows in (("x_local", x_local, n_local), ("x_halo", x_halo, int(i.num_halo))):
        if t is None:
            continue
        if t.dim() != 2 or int(t.shape[1]) < dim:
            raise ValueError(f"{name} must be 2-D with at least {dim} columns, got {tuple(t.shape)}")
        if int(t.shape[0]) < rows:
            raise ValueError(f"{name} has {int(t.shape[0])} rows, the partition needs {rows}")
    if x_halo is None and int(i.num_halo) > 0 and not bags:
        raise ValueError(f"x_halo is missing: the partition has {int(i.num_halo)} halo rows")
    if out is not None:
        if out.dim() != 2 or int(out.shape[0]) < int(i.n_own) or int(out.shape[1]) < dim:
            raise ValueError(f"out must hold at least {int(i.n_own)} x {dim}, got {tuple(out.shape)}")
        if out.device != ref.device:
            raise ValueError("out lives on another device than the tables")


def mgg_aggregate(part: Partition, mode: str, x_local, x_halo=None, *, eps: float = 0.0, out=None,
                  dim: Optional[int] = None, stream=None, out_dtype=None):
    """out[n_own x dim] = Aggregate over N(v) U {v}; fp32, or bf16 (mgg_aggregate_to) when `out` or
    `out_dtype` says so; tensors are torch CUDA tensors."""
    import torch
    dim = int(x_local.shape[1]) if dim is None else dim
    if out is None:
        out = torch.empty((int(part.info.n_own), dim), dtype=out_dtype or torch.float32, device=x_local.device)
    _check_tables(part, x_local, x_halo, out, dim)
    part.reserve(dim)          # the C call allocates nothing; sizing the scratch buffer is a call of its own
    if out.dtype == torch.float32:
        _check(lib().mgg_aggregate(part.handle, _MODE[mode], eps, _torch_dtype_code(x_local), _dev_ptr(x_local),
                                   _dev_ptr(x_halo), dim, _ld(x_local), _dev_ptr(out), _ld(out), _stream(stream)))
    else:
        _check(lib().mgg_aggregate_to(part.handle, _MODE[mode], eps, _torch_dtype_code(x_local), _dev_ptr(x_local),
                                      _dev_ptr(x_halo), dim, _ld(x_local), _torch_dtype_code(out), _dev_ptr(out), _ld(out),
                                      _stream(stream)))
    return out


def mgg_aggregate_static(part: Partition, mode: str, x_local, x_halo=None, *, eps: float = 0.0, out=None,
                         dim: Optional[int] = None, stream=None):
    """mgg_aggregate through the library's fixed scratch array: nothing is allocated or reserved
    (pass `out`, or the output tensor is the one allocation made here, by torch)."""
    import torch
    dim = int(x_local.shape[1]) if dim is None else dim
    if out is None:
        out = torch.empty((int(part.info.n_own), dim), dtype=torch.float32, device=x_local.device)
    _check_tables(part, x_local, x_halo, out, dim)
    _check(lib().mgg_aggregate_static(part.handle, _MODE[mode], eps, _torch_dtype_code(x_local), _dev_ptr(x_local),
                                      _dev_ptr(x_halo), dim, _ld(x_local), _dev_ptr(out), _ld(out), _stream(stream)))
    return out


def mgg_aggregate_scratch_bytes(part: Partition, dim: int) -> int:
    return int(lib().mgg_aggregate_scratch_bytes(part.handle, int(dim)))


def mgg_time_aggregate(part: Partition, mode: str, x_local, x_halo, out, *, eps: float = 0.0, iters: int = 20,
                       dim: Optional[int] = None, stream=None) -> float:
    """Mean milliseconds per mgg_aggregate call, HIP events on the launch stream."""
    dim = int(x_local.shape[1]) if dim is None else dim
    _check_tables(part, x_local, x_halo, out, dim)
    part.reserve(dim)
    ms = C.c_float()
    _check(lib().mgg_time_aggregate(part.handle, _MODE[mode], eps, _torch_dtype_code(x_local), _dev_ptr(x_local),
                                    _dev_ptr(x_halo), dim, _ld(x_local), _dev_ptr(out), _ld(out), _stream(stream),
                                    iters, C.byref(ms)))
    return float(ms.value)


def mgg_probe_gather(table_bytes: int, row_bytes: int = 256, n_gathers: int = 1 << 24, iters: int = 5, seed: int = 7) -> float:
    """Gathered GB/s of random rows from a table of the given size (measurement aid, see mgg.h)."""
    gbs = C.c_double()
    _check(lib().mgg_probe_gather(int(table_bytes), int(row_bytes), int(n_gathers), int(iters), int(seed), C.byref(gbs)))
    return float(gbs.value)


def mgg_update(a, w, bias=None, act: str = "none", *, out=None, out_dtype=None, stream=None):
    """out = act(a @ w + bias) on MFMA."""
    import torch
    n_rows, d_in = int(a.shape[0]), int(a.shape[1])
    d_out = int(w.shape[1])
    if int(w.shape[0]) != d_in or not w.is_contiguous():
        raise ValueError("w must be a contiguous [d_in x d_out] matrix")
    if out is None:
        out = torch.empty((n_rows, d_out), dtype=out_dtype or torch.float32, device=a.device)
    _check(lib().mgg_update(n_rows, _torch_dtype_code(a), _dev_ptr(a), _ld(a), d_in, _torch_dtype_code(w),
                            _dev_ptr(w), _dev_ptr(bias), d_out, _ACT[act], _torch_dtype_code(out), _dev_ptr(out),
                            _ld(out), _stream(stream)))
    return out


def mgg_update_mlp(a, w1, w2, acts=("relu", "none"), biases=(None, None), *, hidden=None, out=None, out_dtype=None,
                   stream=None):
    """out = act2(act1(a @ w1 + b1) @ w2 + b2); one kernel when the shape allows, else two through `hidden`."""
    import torch
    n_rows = int(a.shape[0])
    dims = (C.c_int32 * 3)(int(w1.shape[0]), int(w1.shape[1]), int(w2.shape[1]))
    if int(a.shape[1]) != dims[0] or int(w2.shape[0]) != dims[1] or not (w1.is_contiguous() and w2.is_contiguous()):
        raise ValueError("contiguous [d_in x d_hid] and [d_hid x d_out] matrices expected")
    if out is None:
        out = torch.empty((n_rows, dims[2]), dtype=out_dtype or torch.float32, device=a.device)
    _check(lib().mgg_update_mlp(n_rows, _torch_dtype_code(a), _dev_ptr(a), _ld(a), dims, _torch_dtype_code(w1), _dev_ptr(w1),
                                _dev_ptr(biases[0]), _ACT[acts[0]], _dev_ptr(w2), _dev_ptr(biases[1]), _ACT[acts[1]],
                                _dev_ptr(hidden), 0 if hidden is None else _ld(hidden), _torch_dtype_code(out), _dev_ptr(out),
                                _ld(out), _stream(stream)))
    return out


def _layer_desc(mode, eps, weights, biases, acts, order="agg_first"):
    d = LayerDesc()
    d.order = _ORDER[order]
    d.mode = _MODE[mode]
    d.eps = eps
    d.n_linear = len(weights)
    d.dims[0] = int(weights[0].shape[0])
    for i, w in enumerate(weights):
        if not w.is_contiguous():
            raise ValueError("weights must be contiguous")
        d.dims[i + 1] = int(w.shape[1])
        d.w[i] = w.data_ptr()
        d.bias[i] = None if biases is None or biases[i] is None else biases[i].data_ptr()
        d.act[i] = _ACT[acts[i]]
    d.w_dtype = _torch_dtype_code(weights[0])
    return d


def mgg_layer_workspace_bytes(part: Partition, mode, weights, acts, eps: float = 0.0, biases=None,
                              order: str = "agg_first") -> int:
    d = _layer_desc(mode, eps, weights, biases, acts, order)
    return int(lib().mgg_layer_workspace_bytes(part.handle, C.byref(d)))


def mgg_layer_forward(part: Partition, mode: str, x_local, x_halo, weights, acts, *, eps: float = 0.0,
                      biases=None, workspace=None, out=None, out_dtype=None, stream=None, order: str = "agg_first"):
    """One layer: Aggregate then 1 or 2 Updates (or, order="update_first", the first linear before
    the aggregation), all enqueued on one stream."""
    import torch
    if len(weights) not in (1, 2):
        raise MggError(ERR_INVALID_ARG, "a layer has 1 or 2 linears")
    d = _layer_desc(mode, eps, weights, biases, acts, order)
    need = int(lib().mgg_layer_workspace_bytes(part.handle, C.byref(d)))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x_local.device)
    if out is None:
        out = torch.empty((int(part.info.n_own), int(weights[-1].shape[1])), dtype=out_dtype or torch.float32,
                          device=x_local.device)
    _check_tables(part, x_local, x_halo, None, int(weights[0].shape[0]))
    if int(out.shape[0]) < int(part.info.n_own) or int(out.shape[1]) < int(weights[-1].shape[1]):
        raise ValueError(f"out must hold at least {int(part.info.n_own)} x {int(weights[-1].shape[1])}, got {tuple(out.shape)}")
    _check(lib().mgg_layer_forward(part.handle, C.byref(d), _torch_dtype_code(x_local), _dev_ptr(x_local),
                                   _dev_ptr(x_halo), _ld(x_local), _dev_ptr(workspace), workspace.numel(),
                                   _torch_dtype_code(out), _dev_ptr(out), _ld(out), _stream(stream)))
    return out


# ------------------------------------------------------------------------------- model and tuner
def mgg_model_evaluate(n_local_partitions: int, n_remote_partitions: int, ps: int, dist: int, wpb: int, dim: int,
                       num_units: int = 256, smem_limit_bytes: int = 160 * 1024) -> dict:
    m = Model()
    _check(lib().mgg_model_evaluate(n_local_partitions, n_remote_partitions, Knobs(ps, dist, wpb), dim, num_units,
                                    smem_limit_bytes, C.byref(m)))
    return {"wpw": m.wpw, "smem": m.smem_bytes, "num_warps": m.num_waves, "num_blocks": m.num_blocks,
            "blocks_per_unit": m.blocks_per_unit, "feasible": bool(m.feasible)}


class Tuner:
    """Owner of an ``mgg_tuner_t*`` (propose / report search over ps, dist, wpb)."""

    def __init__(self, ps_max: int = 32, dist_max: int = 16, wpb_max: int = 16):
        h = C.c_void_p()
        _check(lib().mgg_tuner_create(ps_max, dist_max, wpb_max, C.byref(h)))
        self._h = h

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("tuner already destroyed")
        return self._h

    def set_constraint(self, dim: int, smem_limit_bytes: int = 160 * 1024):
        """Bound the search space by the model's shared-memory constraint (before the first trial)."""
        _check(lib().mgg_tuner_set_constraint(self.handle, int(dim), int(smem_limit_bytes)))

    def next(self):
        """The next configuration (ps, dist, wpb) to measure, or None when the search is over."""
        k, done = Knobs(), C.c_int32()
        _check(lib().mgg_tuner_next(self.handle, C.byref(k), C.byref(done)))
        return None if done.value else (k.ps, k.dist, k.wpb)

    def report(self, latency: float):
        _check(lib().mgg_tuner_report(self.handle, float(latency)))

    def result(self):
        k, lat, n = Knobs(), C.c_double(), C.c_int32()
        _check(lib().mgg_tuner_result(self.handle, C.byref(k), C.byref(lat), C.byref(n)))
        return (k.ps, k.dist, k.wpb), lat.value, n.value

    def table(self):
        n = C.c_int32()
        _check(lib().mgg_tuner_table(self.handle, 0, None, None, C.byref(n)))
        ks, lats = (Knobs * max(n.value, 1))(), (C.c_double * max(n.value, 1))()
        _check(lib().mgg_tuner_table(self.handle, n.value, ks, lats, C.byref(n)))
        return [((ks[i].ps, ks[i].dist, ks[i].wpb), lats[i]) for i in range(n.value)]

    def destroy(self):
        if self._h is not None:
            lib().mgg_tuner_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def mgg_tune_aggregate(row_ptr: np.ndarray, col_idx: np.ndarray, num_parts: int, part_id: int, bounds, mode: str,
                       x_local, x_halo, out, tuner: Tuner, *, eps: float = 0.0, iters: int = 10,
                       base_opts: Optional[BuildOpts] = None, stream=None):
    """Runs the search on the GPU; returns ((ps, dist, wpb), best milliseconds)."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    b = None if bounds is None else np.ascontiguousarray(bounds, dtype=np.int64)
    k, ms = Knobs(), C.c_double()
    dim = int(x_local.shape[1])
    _check(lib().mgg_tune_aggregate(row_ptr.size - 1, _np_ptr(row_ptr), _np_ptr(col_idx), num_parts, part_id,
                                    _np_ptr(b), None if base_opts is None else C.byref(base_opts), _MODE[mode], eps,
                                    _torch_dtype_code(x_local), _dev_ptr(x_local), _dev_ptr(x_halo), dim,
                                    _ld(x_local), _dev_ptr(out), _ld(out), _stream(stream), iters, tuner.handle,
                                    C.byref(k), C.byref(ms)))
    return (k.ps, k.dist, k.wpb), ms.value
