"""TEST INFRASTRUCTURE ONLY: ctypes front end of the float64 C oracle (oracle/pc_oracle.c).

Every function takes the block-level DAG arrays of a workload (any object with the attributes
K, n_blocks, root_block, type, n_real, child_ptr, child, param_blk, n_param_blocks, in_var,
in_table, n_vars, n_cats, n_tables) plus the fp32 parameter arrays, and returns float64 results.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        _lib = C.CDLL(path)
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _p(a, typ):
    return None if a is None else a.ctypes.data_as(C.POINTER(typ))


def _chk(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def forward(w, theta, tables, x, mask=None):
    """Eq. (1) in log space.  Returns (lp [B, n_blocks*K], ll [B])."""
    theta = _chk(theta, np.float32); tables = _chk(tables, np.float32); x = _chk(x, np.int32)
    if mask is not None:
        mask = _chk(mask, np.uint8)
    B = x.shape[0]
    lp = np.empty((B, w.n_blocks * w.K), dtype=np.float64)
    ll = np.empty(B, dtype=np.float64)
    rc = lib().orc_forward(
        C.c_int32(w.K), C.c_int32(w.n_blocks), C.c_int32(w.root_block), _p(w.type, C.c_uint8),
        _p(w.child_ptr, C.c_int64), _p(w.child, C.c_int32), _p(w.param_blk, C.c_int32),
        _p(w.in_var, C.c_int32), _p(w.in_table, C.c_int32), C.c_int32(w.n_vars), C.c_int32(w.n_cats),
        _p(theta, C.c_float), _p(tables, C.c_float), _p(x, C.c_int32), _p(mask, C.c_uint8),
        C.c_int32(B), _p(lp, C.c_double), _p(ll, C.c_double))
    if rc != 0:
        raise ValueError("circuit has a cycle")
    return lp, ll


def node_flows(w, theta, lp):
    """Def. 2 node flows.  Returns flow [B, n_blocks*K]."""
    theta = _chk(theta, np.float32)
    B = lp.shape[0]
    flow = np.empty_like(lp)
    rc = lib().orc_node_flows(
        C.c_int32(w.K), C.c_int32(w.n_blocks), C.c_int32(w.root_block), _p(w.type, C.c_uint8),
        _p(w.child_ptr, C.c_int64), _p(w.child, C.c_int32), _p(w.param_blk, C.c_int32),
        _p(theta, C.c_float), C.c_int32(B), _p(lp, C.c_double), _p(flow, C.c_double))
    if rc != 0:
        raise ValueError("circuit has a cycle")
    return flow


def param_flows(w, theta, x, lp, flow, mask=None, theta_flow=None, table_flow=None):
    """Edge flows and input-table flows summed over the batch (added into the given accumulators)."""
    theta = _chk(theta, np.float32); x = _chk(x, np.int32)
    if mask is not None:
        mask = _chk(mask, np.uint8)
    if theta_flow is None:
        theta_flow = np.zeros((w.n_param_blocks + 1, w.K, w.K), dtype=np.float64)
    if table_flow is None:
        table_flow = np.zeros((w.n_tables, w.n_cats, w.K), dtype=np.float64)
    lib().orc_param_flows(
        C.c_int32(w.K), C.c_int32(w.n_blocks), _p(w.type, C.c_uint8),
        _p(w.child_ptr, C.c_int64), _p(w.child, C.c_int32), _p(w.param_blk, C.c_int32),
        _p(w.in_var, C.c_int32), _p(w.in_table, C.c_int32), C.c_int32(w.n_vars), C.c_int32(w.n_cats),
        _p(theta, C.c_float), _p(x, C.c_int32), _p(mask, C.c_uint8), C.c_int32(x.shape[0]),
        _p(lp, C.c_double), _p(flow, C.c_double), _p(theta_flow, C.c_double), _p(table_flow, C.c_double))
    return theta_flow, table_flow


def backward(w, theta, tables, x, mask=None, theta_flow=None, table_flow=None):
    """forward + node flows + parameter flows.  Returns (ll, lp, flow, theta_flow, table_flow)."""
    lp, ll = forward(w, theta, tables, x, mask)
    flow = node_flows(w, theta, lp)
    theta_flow, table_flow = param_flows(w, theta, x, lp, flow, mask, theta_flow, table_flow)
    return ll, lp, flow, theta_flow, table_flow


def em_step(w, theta, tables, theta_flow, table_flow, step=1.0, pseudocount=0.0):
    """In-place EM update of copies of theta / tables; returns (theta, tables) as fp32."""
    theta = np.array(theta, dtype=np.float32, copy=True)
    tables = np.array(tables, dtype=np.float32, copy=True)
    theta_flow = np.array(theta_flow, dtype=np.float64, copy=True)
    table_flow = np.array(table_flow, dtype=np.float64, copy=True)
    lib().orc_em_step(
        C.c_int32(w.K), C.c_int32(w.n_blocks), _p(w.type, C.c_uint8), _p(w.n_real, C.c_int32),
        _p(w.child_ptr, C.c_int64), _p(w.child, C.c_int32), _p(w.param_blk, C.c_int32),
        C.c_int32(w.n_param_blocks), C.c_int32(w.n_cats), C.c_int32(w.n_tables),
        _p(theta, C.c_float), _p(tables, C.c_float), _p(theta_flow, C.c_double), _p(table_flow, C.c_double),
        C.c_double(step), C.c_double(pseudocount))
    return theta, tables
