"""ctypes front-end of the CPU oracle (``mgg_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by
the ``cpu_baseline`` leg of ``bench.py``; never by the product package.  It shares no
code with the HIP library and does not import it.  All arithmetic lives in the C file
(double precision); this module only marshals numpy arrays.

The paper sections each routine follows are cited in ``mgg_oracle.c``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mgg_oracle.c")
_LIB = os.path.join(_HERE, "libmgg_oracle.so")

F32, BF16, F64 = 0, 1, 2
GCN, GIN = 0, 1
ACT_NONE, ACT_RELU = 0, 1
_MODE = {"gcn": GCN, "gin": GIN}
_ACT = {"none": ACT_NONE, "relu": ACT_RELU, "softmax": 2}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.mgg_oracle_groups.restype = C.c_int64
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def num_threads() -> int:
    return int(lib().mgg_oracle_num_threads())


def _table(x: np.ndarray):
    """-> (contiguous array, dtype code, leading dimension)."""
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        code = F32
    elif x.dtype == np.float64:
        code = F64
    elif x.dtype == np.uint16:
        code = BF16
    else:
        raise TypeError(f"unsupported table dtype {x.dtype}")
    return x, code, (x.shape[1] if x.ndim == 2 else 1)


def degrees(row_ptr, col) -> np.ndarray:
    row_ptr, col = _i64(row_ptr), _i32(col)
    n = row_ptr.size - 1
    deg = np.empty(n, dtype=np.int32)
    _check(lib().mgg_oracle_degrees(C.c_int64(n), _p(row_ptr), _p(col), _p(deg)), "degrees")
    return deg


def build_partition(row_ptr, col, parts: int, part_id: int, bounds) -> dict:
    """Local CSR, remote CSR, halo list, owner spans and degrees of one node range."""
    row_ptr, col, bounds = _i64(row_ptr), _i32(col), _i64(bounds)
    n = row_ptr.size - 1
    nl, nr, nh = C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib().mgg_oracle_partition_sizes(C.c_int64(n), _p(row_ptr), _p(col), C.c_int32(parts),
                                            C.c_int32(part_id), _p(bounds),
                                            C.byref(nl), C.byref(nr), C.byref(nh)), "partition_sizes")
    lb, ub = int(bounds[part_id]), int(bounds[part_id + 1])
    n_own = ub - lb
    out = {
        "lb": lb, "ub": ub, "n_own": n_own,
        "local_row_ptr": np.zeros(n_own + 1, dtype=np.int64),
        "local_col": np.zeros(nl.value, dtype=np.int32),
        "remote_row_ptr": np.zeros(n_own + 1, dtype=np.int64),
        "remote_col": np.zeros(nr.value, dtype=np.int32),
        "halo_gid": np.zeros(nh.value, dtype=np.int32),
        "halo_peer_ptr": np.zeros(parts + 1, dtype=np.int64),
        "deg_own": np.zeros(n_own, dtype=np.int32),
        "deg_halo": np.zeros(nh.value, dtype=np.int32),
    }
    _check(lib().mgg_oracle_partition_fill(
        C.c_int64(n), _p(row_ptr), _p(col), C.c_int32(parts), C.c_int32(part_id), _p(bounds),
        _p(out["local_row_ptr"]), _p(out["local_col"]), _p(out["remote_row_ptr"]),
        _p(out["remote_col"]), _p(out["halo_gid"]), _p(out["halo_peer_ptr"]),
        _p(out["deg_own"]), _p(out["deg_halo"])), "partition_fill")
    return out


def neighbor_groups(row_ptr, ps: int):
    """(row, start, end) of every group of <= ps neighbours, rows in order."""
    row_ptr = _i64(row_ptr)
    n_rows = row_ptr.size - 1
    cnt = lib().mgg_oracle_groups(C.c_int64(n_rows), _p(row_ptr), C.c_int32(ps), None, None, None)
    if cnt < 0:
        raise ValueError("oracle groups: bad arguments")
    row = np.zeros(cnt, dtype=np.int32)
    start = np.zeros(cnt, dtype=np.int64)
    end = np.zeros(cnt, dtype=np.int64)
    lib().mgg_oracle_groups(C.c_int64(n_rows), _p(row_ptr), C.c_int32(ps), _p(row), _p(start), _p(end))
    return row, start, end


def aggregate(row_ptr, col, mode: str, x_local: np.ndarray, *, lb: int = 0, ub: Optional[int] = None,
              x_halo: Optional[np.ndarray] = None, halo_gid: Optional[np.ndarray] = None,
              eps: float = 0.0, dim: Optional[int] = None,
              rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Aggregate for the owned rows [lb, ub) (default: the whole graph) -> float64."""
    row_ptr, col = _i64(row_ptr), _i32(col)
    n = row_ptr.size - 1
    ub = n if ub is None else ub
    xl, code, ld = _table(x_local)
    dim = ld if dim is None else dim
    xh = hg = None
    nh = 0
    if x_halo is not None and halo_gid is not None and len(halo_gid):
        xh, code_h, ld_h = _table(x_halo)
        if code_h != code or ld_h != ld:
            raise TypeError("halo table must match the local table's dtype and width")
        hg = _i32(halo_gid)
        nh = hg.size
    sel = None if rows is None else _i64(rows)
    n_out = (ub - lb) if sel is None else sel.size
    out = np.zeros((n_out, dim), dtype=np.float64)
    _check(lib().mgg_oracle_aggregate(
        C.c_int64(n), _p(row_ptr), _p(col), C.c_int64(lb), C.c_int64(ub),
        C.c_int32(_MODE[mode]), C.c_double(eps), C.c_int32(code), _p(xl), _p(xh), _p(hg),
        C.c_int64(nh), C.c_int32(dim), C.c_int64(ld), _p(sel),
        C.c_int64(0 if sel is None else sel.size), _p(out)), "aggregate")
    return out


def bag_sum(bag_ptr, bag_idx, table: np.ndarray) -> np.ndarray:
    """Sum of the looked-up rows of every bag over the whole table -> float64 [num_bags x dim]."""
    bag_ptr, bag_idx = _i64(bag_ptr), _i32(bag_idx)
    tab, code, ld = _table(table)
    nb = bag_ptr.size - 1
    out = np.zeros((nb, ld), dtype=np.float64)
    _check(lib().mgg_oracle_bag_sum(C.c_int64(nb), _p(bag_ptr), _p(bag_idx), C.c_int64(table.shape[0]), C.c_int32(code), _p(tab),
                                    C.c_int64(ld), C.c_int32(ld), _p(out)), "bag_sum")
    return out


def to_f64(t: np.ndarray) -> np.ndarray:
    """Exact widening of f32 / bf16-bit / f64 arrays to float64."""
    t = np.asarray(t)
    if t.dtype == np.uint16:
        return (t.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return t.astype(np.float64)


def update(a: np.ndarray, w: np.ndarray, bias: Optional[np.ndarray] = None, act: str = "none") -> np.ndarray:
    """act(a @ w + bias) by triple loop in float64."""
    a = np.ascontiguousarray(to_f64(a))
    w = np.ascontiguousarray(to_f64(w))
    b = None if bias is None else np.ascontiguousarray(to_f64(bias))
    n_rows, d_in = a.shape
    d_out = w.shape[1]
    if w.shape[0] != d_in:
        raise ValueError("shape mismatch")
    out = np.zeros((n_rows, d_out), dtype=np.float64)
    _check(lib().mgg_oracle_update(C.c_int64(n_rows), _p(a), C.c_int64(d_in), C.c_int32(d_in), _p(w),
                                   _p(b), C.c_int32(d_out), C.c_int32(_ACT[act]), _p(out),
                                   C.c_int64(d_out)), "update")
    return out


def layer_forward(row_ptr, col, mode: str, x_local, weights, acts, *, biases=None, eps: float = 0.0,
                  lb: int = 0, ub: Optional[int] = None, x_halo=None, halo_gid=None,
                  rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """Aggregate, then one Update per weight matrix (GCN: one; GIN MLP: two)."""
    h = aggregate(row_ptr, col, mode, x_local, lb=lb, ub=ub, x_halo=x_halo, halo_gid=halo_gid,
                  eps=eps, rows=rows)
    for i, w in enumerate(weights):
        h = update(h, w, None if biases is None else biases[i], acts[i])
    return h


def split_edge_balanced(row_ptr, parts: int) -> np.ndarray:
    row_ptr = _i64(row_ptr)
    n = row_ptr.size - 1
    bounds = np.zeros(parts + 1, dtype=np.int64)
    _check(lib().mgg_oracle_split_edge_balanced(C.c_int64(n), _p(row_ptr), C.c_int32(parts),
                                                _p(bounds)), "split")
    return bounds
