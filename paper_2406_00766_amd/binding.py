"""Thin ctypes binding of libpc (argument marshalling only; every step of the path runs in the library).

Function names mirror the C ABI declared in include/pc.h.  Device buffers are torch tensors (or raw
integer addresses); torch is used for device memory and streams only.  There is no CPU fallback: if
libpc.so is missing, importing a function from here raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpc.so")

PC_OK = 0
STATUS_NAMES = ["PC_OK", "PC_ERR_ARG", "PC_ERR_CYCLE", "PC_ERR_NOT_ALTERNATING", "PC_ERR_NOT_BLOCK_SPARSE",
                "PC_ERR_TIE", "PC_ERR_TOO_LARGE", "PC_ERR_WORKSPACE", "PC_ERR_STATE", "PC_ERR_HIP"]


class PcError(RuntimeError):
    def __init__(self, status: int, message: str):
        self.status = status
        self.status_name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{self.status_name}: {message}")


class pc_dag(C.Structure):
    _fields_ = [("K", C.c_int32), ("n_blocks", C.c_int32), ("root_block", C.c_int32),
                ("type", C.POINTER(C.c_uint8)), ("n_real", C.POINTER(C.c_int32)),
                ("child_ptr", C.POINTER(C.c_int64)), ("child", C.POINTER(C.c_int32)),
                ("param_blk", C.POINTER(C.c_int32)), ("n_param_blocks", C.c_int32),
                ("in_var", C.POINTER(C.c_int32)), ("in_table", C.POINTER(C.c_int32)),
                ("n_vars", C.c_int32), ("n_cats", C.c_int32), ("n_tables", C.c_int32),
                ("max_groups", C.c_int32), ("tol_permille", C.c_int32), ("product_scratch", C.c_int32)]


class pc_sizes(C.Structure):
    _fields_ = [("K", C.c_int32), ("n_blocks", C.c_int32), ("n_layers", C.c_int32),
                ("n_rows", C.c_int64), ("theta_len", C.c_int64), ("tables_len", C.c_int64),
                ("n_vars", C.c_int32), ("n_cats", C.c_int32), ("n_tables", C.c_int32)]


class pc_layer_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("depth", C.c_int32), ("n_fwd_groups", C.c_int32), ("n_bwd_groups", C.c_int32)]


class pc_group_desc(C.Structure):
    _fields_ = [("n_rows", C.c_int32), ("width", C.c_int32),
                ("ids", C.c_void_p), ("nbr", C.c_void_p), ("par", C.c_void_p)]


class pc_ws_layout(C.Structure):
    _fields_ = [("stride", C.c_int64), ("l_offset", C.c_size_t), ("f_offset", C.c_size_t),
                ("n_offset", C.c_size_t), ("r_offset", C.c_size_t), ("total_bytes", C.c_size_t), ("l_rows", C.c_int64)]


class pc_profile(C.Structure):
    _fields_ = [("n_classes", C.c_int32), ("launches", C.c_int64 * 16), ("ms", C.c_double * 16),
                ("bf16_launches", C.c_int64 * 16)]


EXPORTS = ["pc_compile", "pc_compile_host", "pc_destroy", "pc_last_error", "pc_get_sizes", "pc_get_layer",
           "pc_get_group", "pc_copy_group", "pc_workspace_layout", "pc_workspace_bytes", "pc_forward",
           "pc_forward_static", "pc_backward", "pc_em_step", "pc_profile_enable", "pc_profile_read", "pc_kernel_class_name",
           "pc_measure_copy", "pc_measure_mfma_f32", "pc_collapse", "pc_collapsed_dag", "pc_collapsed_theta",
           "pc_collapsed_block_map", "pc_collapsed_destroy", "pc_order_for_scratch"]

_lib = None


def lib():
    """Load libpc.so (built by paper_2406_00766_amd/build.py).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2406_00766_amd.build` "
                                    "(or __graft_entry__.build())")
        L = C.CDLL(LIB_PATH)
        L.pc_last_error.restype = C.c_char_p
        L.pc_destroy.restype = None
        L.pc_destroy.argtypes = [C.c_void_p]
        L.pc_compile.argtypes = [C.POINTER(pc_dag), C.c_void_p, C.POINTER(C.c_void_p)]
        L.pc_compile_host.argtypes = [C.POINTER(pc_dag), C.POINTER(C.c_void_p)]
        L.pc_get_sizes.argtypes = [C.c_void_p, C.POINTER(pc_sizes)]
        L.pc_get_layer.argtypes = [C.c_void_p, C.c_int32, C.POINTER(pc_layer_desc)]
        L.pc_get_group.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(pc_group_desc)]
        L.pc_copy_group.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.pc_workspace_layout.argtypes = [C.c_void_p, C.c_int32, C.POINTER(pc_ws_layout)]
        L.pc_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_size_t)]
        L.pc_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                 C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.pc_forward_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                        C.c_void_p, C.c_void_p]
        L.pc_backward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                  C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]
        L.pc_em_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_float, C.c_float, C.c_void_p]
        L.pc_profile_enable.argtypes = [C.c_void_p, C.c_int32]
        L.pc_profile_read.argtypes = [C.c_void_p, C.POINTER(pc_profile)]
        L.pc_kernel_class_name.argtypes = [C.c_int32]
        L.pc_kernel_class_name.restype = C.c_char_p
        L.pc_measure_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
        L.pc_measure_mfma_f32.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
        L.pc_collapse.argtypes = [C.POINTER(pc_dag), C.c_void_p, C.POINTER(C.c_void_p)]
        L.pc_order_for_scratch.argtypes = [C.POINTER(pc_dag), C.POINTER(C.c_void_p)]
        L.pc_collapsed_dag.argtypes = [C.c_void_p]
        L.pc_collapsed_dag.restype = C.POINTER(pc_dag)
        L.pc_collapsed_theta.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
        L.pc_collapsed_theta.restype = C.POINTER(C.c_float)
        L.pc_collapsed_block_map.argtypes = [C.c_void_p]
        L.pc_collapsed_block_map.restype = C.POINTER(C.c_int32)
        L.pc_collapsed_destroy.argtypes = [C.c_void_p]
        L.pc_collapsed_destroy.restype = None
        _lib = L
    return _lib


def _check(status: int):
    if status != PC_OK:
        raise PcError(status, (lib().pc_last_error() or b"").decode())


def _ptr(t):
    """Device address of a torch tensor / raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_dag(w):
    """Marshal a workload-like object (see workloads.Workload) into a pc_dag; returns (dag, keepalive)."""
    arrs = dict(
        type=np.ascontiguousarray(w.type, dtype=np.uint8), n_real=np.ascontiguousarray(w.n_real, dtype=np.int32),
        child_ptr=np.ascontiguousarray(w.child_ptr, dtype=np.int64), child=np.ascontiguousarray(w.child, dtype=np.int32),
        param_blk=np.ascontiguousarray(w.param_blk, dtype=np.int32), in_var=np.ascontiguousarray(w.in_var, dtype=np.int32),
        in_table=np.ascontiguousarray(w.in_table, dtype=np.int32))
    d = pc_dag()
    d.K, d.n_blocks, d.root_block = int(w.K), int(w.n_blocks), int(w.root_block)
    d.type = arrs["type"].ctypes.data_as(C.POINTER(C.c_uint8))
    d.n_real = arrs["n_real"].ctypes.data_as(C.POINTER(C.c_int32))
    d.child_ptr = arrs["child_ptr"].ctypes.data_as(C.POINTER(C.c_int64))
    d.child = arrs["child"].ctypes.data_as(C.POINTER(C.c_int32))
    d.param_blk = arrs["param_blk"].ctypes.data_as(C.POINTER(C.c_int32))
    d.n_param_blocks = int(w.n_param_blocks)
    d.in_var = arrs["in_var"].ctypes.data_as(C.POINTER(C.c_int32))
    d.in_table = arrs["in_table"].ctypes.data_as(C.POINTER(C.c_int32))
    d.n_vars, d.n_cats, d.n_tables = int(w.n_vars), int(w.n_cats), int(w.n_tables)
    d.max_groups, d.tol_permille = int(w.max_groups), int(w.tol_permille)
    d.product_scratch = int(getattr(w, "product_scratch", 0))
    return d, arrs


def pc_compile(w, stream=None, host_only: bool = False) -> int:
    """Returns the opaque circuit handle (an integer address)."""
    d, keep = make_dag(w)
    out = C.c_void_p()
    if host_only:
        _check(lib().pc_compile_host(C.byref(d), C.byref(out)))
    else:
        _check(lib().pc_compile(C.byref(d), _stream(stream), C.byref(out)))
    del keep
    return out.value


def pc_collapse(w):
    """Footnote to Def. 2: the alternating form of a DAG with consecutive sum / sum or product / product blocks.
    Returns a copy of the workload-like object `w` with the rewritten DAG arrays, `theta` and `block_map`."""
    return _rewritten(w, collapse=True)


def pc_order_for_scratch(w):
    """Sec. 5, product-scratch mode: a copy of `w` with its blocks renumbered (input and sum blocks first, product
    blocks grouped by the sum layer that reads them, copied where sum layers of several depths read them),
    `product_scratch` set and `block_map` (old id -> new id)."""
    return _rewritten(w, collapse=False)


def _rewritten(w, collapse: bool):
    import copy
    d, keep = make_dag(w)
    theta = np.ascontiguousarray(w.theta, dtype=np.float32)
    out = C.c_void_p()
    if collapse:
        _check(lib().pc_collapse(C.byref(d), theta.ctypes.data, C.byref(out)))
    else:
        _check(lib().pc_order_for_scratch(C.byref(d), C.byref(out)))
    try:
        nd = lib().pc_collapsed_dag(out).contents
        n, ne = int(nd.n_blocks), int(nd.child_ptr[nd.n_blocks])
        r = copy.copy(w)
        r.n_blocks, r.root_block, r.n_param_blocks = n, int(nd.root_block), int(nd.n_param_blocks)
        r.type = np.ctypeslib.as_array(nd.type, (n,)).copy()
        r.n_real = np.ctypeslib.as_array(nd.n_real, (n,)).copy()
        r.child_ptr = np.ctypeslib.as_array(nd.child_ptr, (n + 1,)).copy()
        r.child = np.ctypeslib.as_array(nd.child, (max(ne, 1),))[:ne].copy()
        r.param_blk = np.ctypeslib.as_array(nd.param_blk, (max(ne, 1),))[:ne].copy()
        r.in_var = np.ctypeslib.as_array(nd.in_var, (n,)).copy()
        r.in_table = np.ctypeslib.as_array(nd.in_table, (n,)).copy()
        if collapse:
            ln = C.c_int64()
            tp = lib().pc_collapsed_theta(out, C.byref(ln))
            r.theta = np.ctypeslib.as_array(tp, (int(ln.value),)).copy().reshape(-1, w.K, w.K)
        else:
            r.product_scratch = 1
        r.block_map = np.ctypeslib.as_array(lib().pc_collapsed_block_map(out), (int(w.n_blocks),)).copy()
    finally:
        lib().pc_collapsed_destroy(out)
    del keep
    return r


def pc_destroy(handle: int):
    lib().pc_destroy(handle)


def pc_get_sizes(handle: int) -> pc_sizes:
    s = pc_sizes()
    _check(lib().pc_get_sizes(handle, C.byref(s)))
    return s


def pc_get_layer(handle: int, layer: int) -> pc_layer_desc:
    d = pc_layer_desc()
    _check(lib().pc_get_layer(handle, layer, C.byref(d)))
    return d


def pc_get_group(handle: int, layer: int, direction: int, group: int) -> pc_group_desc:
    g = pc_group_desc()
    _check(lib().pc_get_group(handle, layer, direction, group, C.byref(g)))
    return g


def pc_copy_group(handle: int, layer: int, direction: int, group: int):
    """(ids [R], nbr [R, W], par [R, W]) as int32 numpy arrays."""
    g = pc_get_group(handle, layer, direction, group)
    ids = np.empty(g.n_rows, dtype=np.int32)
    nbr = np.empty((g.n_rows, g.width), dtype=np.int32)
    par = np.empty((g.n_rows, g.width), dtype=np.int32)
    _check(lib().pc_copy_group(handle, layer, direction, group, ids.ctypes.data, nbr.ctypes.data, par.ctypes.data))
    return ids, nbr, par


def pc_workspace_layout(handle: int, B: int) -> pc_ws_layout:
    lay = pc_ws_layout()
    _check(lib().pc_workspace_layout(handle, B, C.byref(lay)))
    return lay


def pc_workspace_bytes(handle: int, B: int) -> int:
    n = C.c_size_t()
    _check(lib().pc_workspace_bytes(handle, B, C.byref(n)))
    return int(n.value)


def pc_forward(handle, theta, tables, x, mask, B, workspace, workspace_bytes, ll, stream=None):
    _check(lib().pc_forward(handle, _ptr(theta), _ptr(tables), _ptr(x), _ptr(mask), int(B), _ptr(workspace),
                            int(workspace_bytes), _ptr(ll), _stream(stream)))


PC_STATIC_SCRATCH_BYTES = 64 << 20


def pc_forward_static(handle, theta, tables, x, mask, B, ll, stream=None):
    _check(lib().pc_forward_static(handle, _ptr(theta), _ptr(tables), _ptr(x), _ptr(mask), int(B), _ptr(ll),
                                   _stream(stream)))


def pc_backward(handle, theta, tables, x, mask, B, workspace, workspace_bytes, theta_flow, table_flow, stream=None):
    _check(lib().pc_backward(handle, _ptr(theta), _ptr(tables), _ptr(x), _ptr(mask), int(B), _ptr(workspace),
                             int(workspace_bytes), _ptr(theta_flow), _ptr(table_flow), _stream(stream)))


def pc_em_step(handle, theta, tables, theta_flow, table_flow, step, pseudocount, stream=None):
    _check(lib().pc_em_step(handle, _ptr(theta), _ptr(tables), _ptr(theta_flow), _ptr(table_flow),
                            float(step), float(pseudocount), _stream(stream)))


def pc_profile_enable(handle: int, on: bool):
    _check(lib().pc_profile_enable(handle, 1 if on else 0))


def pc_profile_read(handle: int, with_bf16: bool = False) -> dict:
    """{class name: (launches, total ms)} since pc_profile_enable; with_bf16 adds the launches that ran as bf16-split
    products as a third element."""
    p = pc_profile()
    _check(lib().pc_profile_read(handle, C.byref(p)))
    if with_bf16:
        return {lib().pc_kernel_class_name(i).decode(): (int(p.launches[i]), float(p.ms[i]), int(p.bf16_launches[i]))
                for i in range(p.n_classes)}
    return {lib().pc_kernel_class_name(i).decode(): (int(p.launches[i]), float(p.ms[i])) for i in range(p.n_classes)}


def pc_measure_copy(src, dst, nbytes: int, reps: int = 5, stream=None) -> float:
    """GB/s (read + written) of a plain streaming copy between two device buffers."""
    out = C.c_double()
    _check(lib().pc_measure_copy(_ptr(src), _ptr(dst), int(nbytes), int(reps), _stream(stream), C.byref(out)))
    return float(out.value)


def pc_measure_mfma_f32(out_buf, out_bytes: int, reps: int = 5, stream=None) -> float:
    """TFLOP/s of a register-only fp32 MFMA loop; out_buf: device buffer of at least 2 MiB."""
    out = C.c_double()
    _check(lib().pc_measure_mfma_f32(_ptr(out_buf), int(out_bytes), int(reps), _stream(stream), C.byref(out)))
    return float(out.value)


def compiled_tables(handle: int) -> list[dict]:
    """All layers with their groups copied to host: [{kind, depth, fwd: [(ids, nbr, par)], bwd: [...]}]."""
    out = []
    for li in range(pc_get_sizes(handle).n_layers):
        d = pc_get_layer(handle, li)
        out.append({"kind": d.kind, "depth": d.depth,
                    "fwd": [pc_copy_group(handle, li, 0, g) for g in range(d.n_fwd_groups)],
                    "bwd": [pc_copy_group(handle, li, 1, g) for g in range(d.n_bwd_groups)]})
    return out


class Circuit:
    """Convenience owner of a handle plus device copies of one workload's arrays (tests / benchmark)."""

    def __init__(self, w, device="cuda:0"):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.handle = pc_compile(w)
        self.sizes = pc_get_sizes(self.handle)
        self.K = w.K
        self.theta = torch.from_numpy(np.ascontiguousarray(w.theta, dtype=np.float32).reshape(-1)).to(self.device)
        self.tables = torch.from_numpy(np.ascontiguousarray(w.tables, dtype=np.float32).reshape(-1)).to(self.device)
        assert self.theta.numel() == self.sizes.theta_len and self.tables.numel() == self.sizes.tables_len
        self.theta_flow = torch.zeros_like(self.theta)
        self.table_flow = torch.zeros_like(self.tables)
        self._ws = None
        self._ws_B = 0
        self.x = self.mask = self.ll = None
        self.B = 0

    def close(self):
        if self.handle:
            pc_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_batch(self, x, mask=None):
        torch = self.torch
        self.x = torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(self.device)
        self.mask = None if mask is None else torch.from_numpy(np.ascontiguousarray(mask, dtype=np.uint8)).to(self.device)
        self.B = int(x.shape[0])
        need = pc_workspace_bytes(self.handle, self.B)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        self.ll = torch.empty(self.B, dtype=torch.float32, device=self.device)

    def forward(self):
        pc_forward(self.handle, self.theta, self.tables, self.x, self.mask, self.B, self._ws, self._ws.numel(), self.ll)
        return self.ll

    def backward(self, theta_flow=True, table_flow=True):
        pc_backward(self.handle, self.theta, self.tables, self.x, self.mask, self.B, self._ws, self._ws.numel(),
                    self.theta_flow if theta_flow else None, self.table_flow if table_flow else None)

    def em_step(self, step=1.0, pseudocount=0.0):
        pc_em_step(self.handle, self.theta, self.tables, self.theta_flow, self.table_flow, step, pseudocount)

    def node_buffers(self):
        """(l, F, R) float32 views of the workspace: l, F are [n_rows, stride] (row = compiled node offset),
        R is [n_blocks + 1, stride]; the log-probability of row n is R[n // K] + l[n]."""
        lay = pc_workspace_layout(self.handle, self.B)
        n = self.sizes.n_rows * lay.stride
        nb = (self.sizes.n_blocks + 1) * lay.stride
        f32 = self.torch.float32
        l = self._ws[lay.l_offset:lay.l_offset + 4 * lay.l_rows * lay.stride].view(f32).view(lay.l_rows, lay.stride)
        F = self._ws[lay.f_offset:lay.f_offset + 4 * lay.l_rows * lay.stride].view(f32).view(lay.l_rows, lay.stride)
        R = self._ws[lay.r_offset:lay.r_offset + 4 * nb].view(f32).view(self.sizes.n_blocks + 1, lay.stride)
        return l, F, R
