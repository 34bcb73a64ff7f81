"""Thin ctypes binding of liblwp.so (the C ABI in include/lwp.h).

Argument marshalling only: every step of the search runs inside the library's
HIP kernels.  PyTorch supplies device memory (int32 CUDA tensors) and the
stream handle, nothing else.  There is no CPU fallback: if the library is not
built, or no GPU is present, calls fail loudly.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblwp.so")

OK, E_INVAL, E_GRAPH, E_NOT_REDUCIBLE, E_OVERFLOW, E_NOMEM, E_HIP, E_TOO_LARGE = 0, -1, -2, -3, -4, -5, -6, -7
NOALLOC_MAX_BATCH = 4096
SCHEDULE_ROUNDS, SCHEDULE_LEFT_FOLD, SCHEDULE_NONE = 0, 1, 2
UNDO_STORED, UNDO_RECOMPUTE = 0, 1

EXPORTED = [
    "lwp_create", "lwp_destroy", "lwp_last_error", "lwp_status_string", "lwp_synchronize", "lwp_set_option",
    "lwp_eliminate_node", "lwp_eliminate_node_bounded", "lwp_eliminate_node_noalloc", "lwp_eliminate_edge", "lwp_plan_graph", "lwp_search_graph",
    "lwp_search_workspace_bytes", "lwp_search_graph_ex", "lwp_search_workspace_bytes_ex",
    "lwp_search_graph_ragged", "lwp_search_workspace_bytes_ragged", "lwp_build_cost_tables",
    "lwp_build_cost_tables_ragged", "lwp_build_cost_tables_graph", "lwp_enumerate_configs",
    "lwp_search_plan_create", "lwp_search_plan_run", "lwp_search_plan_destroy", "lwp_measure_valu_rate",
    "lwp_profile_enable", "lwp_profile_reset", "lwp_profile_read",
]

STEP_DTYPE = np.dtype([("kind", "<i4"), ("j", "<i4"), ("i", "<i4"), ("k", "<i4"),
                       ("e1", "<i4"), ("e2", "<i4"), ("round", "<i4")])
LAYER_DTYPE = np.dtype([(n, "<i4") for n in ("kind", "N", "Cin", "Hin", "Win", "Cout", "Hout", "Wout",
                                             "kh", "kw", "sh", "sw", "ph", "pw")])
CONFIG_DTYPE = np.dtype([(n, "<i4") for n in ("n", "h", "w", "c", "dev_offset", "pad")])
MACHINE_DTYPE = np.dtype([(n, "<i4") for n in ("n_devices", "flop_per_ns", "byte_per_ns", "invalid_cost")])


class Profile(ctypes.Structure):
    _fields_ = [("node_launches", ctypes.c_int64), ("node_cell_updates", ctypes.c_int64),
                ("node_ms", ctypes.c_double), ("edge_launches", ctypes.c_int64),
                ("edge_cells", ctypes.c_int64), ("edge_ms", ctypes.c_double),
                ("keyed_launches", ctypes.c_int64), ("products_keyed", ctypes.c_int64),
                ("products_keyed_row", ctypes.c_int64), ("products_plain", ctypes.c_int64),
                ("products_value", ctypes.c_int64)]


class DeviceGraph(ctypes.Structure):
    _fields_ = [("n_devices", ctypes.c_int32), ("flop_per_ns", ctypes.c_int32), ("invalid_cost", ctypes.c_int32),
                ("pad", ctypes.c_int32), ("bandwidth", ctypes.c_void_p)]


class LwpError(RuntimeError):
    def __init__(self, code, what, detail=""):
        super().__init__(f"{what}: status {code}" + (f" ({detail})" if detail else ""))
        self.code = code


_lib = None


def load():
    """Loads liblwp.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_1802_04924_amd.build` "
                           "(or __graft_entry__.build()) first")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i32p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)
    lib.lwp_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, vp]
    lib.lwp_destroy.argtypes = [vp]
    lib.lwp_destroy.restype = None
    lib.lwp_last_error.argtypes = [vp]
    lib.lwp_last_error.restype = ctypes.c_char_p
    lib.lwp_status_string.argtypes = [ctypes.c_int]
    lib.lwp_status_string.restype = ctypes.c_char_p
    lib.lwp_synchronize.argtypes = [vp]
    lib.lwp_set_option.argtypes = [vp, i32, i32]
    lib.lwp_eliminate_node.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.lwp_eliminate_node_bounded.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.lwp_eliminate_node_noalloc.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.lwp_eliminate_edge.argtypes = [vp, i32, i32, i32, vp, vp, vp]
    lib.lwp_plan_graph.argtypes = [i32, i32, vp, i32, vp, i32p, i32p, i32p]
    lib.lwp_search_graph.argtypes = [vp, i32, i32, vp, i32, vp, vp, vp, i32, i32p, vp]
    lib.lwp_search_workspace_bytes.argtypes = [i32, i32, vp, i32, i32]
    lib.lwp_search_workspace_bytes.restype = ctypes.c_size_t
    lib.lwp_search_graph_ex.argtypes = [vp, i32, i32, vp, i32, vp, vp, vp, i32, i32, i32p, vp]
    lib.lwp_search_workspace_bytes_ex.argtypes = [i32, i32, vp, i32, i32, i32]
    lib.lwp_search_workspace_bytes_ex.restype = ctypes.c_size_t
    lib.lwp_search_graph_ragged.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, i32, i32, i32p, vp]
    lib.lwp_search_workspace_bytes_ragged.argtypes = [i32, i32, vp, vp, i32, i32]
    lib.lwp_search_workspace_bytes_ragged.restype = ctypes.c_size_t
    lib.lwp_build_cost_tables.argtypes = [vp, vp, i32, vp, i32, vp, i32, vp, vp, vp, vp]
    lib.lwp_build_cost_tables_ragged.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.lwp_build_cost_tables_graph.argtypes = [vp, vp, i32, vp, i32, vp, vp, ctypes.POINTER(DeviceGraph), vp, vp, vp, vp]
    lib.lwp_enumerate_configs.argtypes = [vp, i32, vp, i32, i32p]
    lib.lwp_search_plan_create.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, i32, ctypes.POINTER(vp)]
    lib.lwp_search_plan_run.argtypes = [vp, i32p, vp]
    lib.lwp_search_plan_destroy.argtypes = [vp]
    lib.lwp_search_plan_destroy.restype = None
    lib.lwp_measure_valu_rate.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.lwp_profile_enable.argtypes = [vp, i32]
    lib.lwp_profile_reset.argtypes = [vp]
    lib.lwp_profile_read.argtypes = [vp, ctypes.POINTER(Profile)]
    _lib = lib
    return lib


def _np_i32(a, shape=None):
    if not (type(a) is np.ndarray and a.dtype == np.int32 and a.flags.c_contiguous):
        a = np.ascontiguousarray(a, dtype=np.int32)
    if shape is not None:
        a = a.reshape(shape)
    return a


def _ptr(a):
    """Address of a numpy array's data (a search of tens of microseconds feels `a.ctypes.data`, which builds a helper object)."""
    try:
        return ctypes.addressof(ctypes.c_char.from_buffer(a))
    except (TypeError, ValueError):           # read-only or empty
        return a.ctypes.data


def _result_buffer(n):
    """int32 [n] the library writes a strategy into: (numpy view, address)."""
    buf = (ctypes.c_int32 * n)()
    return np.frombuffer(buf, dtype=np.int32), ctypes.addressof(buf)


def plan_graph(n_nodes, edges, schedule=SCHEDULE_ROUNDS):
    """Host-only elimination schedule: dict(steps, n_rounds, n_residual_nodes)."""
    lib = load()
    edges = _np_i32(edges, (-1, 2))
    steps = np.zeros(max(len(edges), 1), STEP_DTYPE)
    ns, nr, nk = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib.lwp_plan_graph(n_nodes, len(edges), edges.ctypes.data, int(schedule), steps.ctypes.data,
                            ctypes.byref(ns), ctypes.byref(nr), ctypes.byref(nk))
    if rc:
        raise LwpError(rc, "plan_graph", lib.lwp_status_string(rc).decode())
    return {"steps": steps[:ns.value], "n_rounds": nr.value, "n_residual_nodes": nk.value}


def search_workspace_bytes(n_nodes, edges, C, schedule=SCHEDULE_ROUNDS, undo=UNDO_STORED) -> int:
    lib = load()
    edges = _np_i32(edges, (-1, 2))
    return int(lib.lwp_search_workspace_bytes_ex(n_nodes, len(edges), edges.ctypes.data, C, int(schedule), int(undo)))


def enumerate_configs(layer, n_devices) -> np.ndarray:
    """Host-only: configurations of one layer (int32 [C][6]) on a machine of n_devices."""
    lib = load()
    layer = _np_i32(layer, (14,))
    n = ctypes.c_int32(0)
    rc = lib.lwp_enumerate_configs(layer.ctypes.data, int(n_devices), None, 0, ctypes.byref(n))
    if rc:
        raise LwpError(rc, "enumerate_configs", lib.lwp_status_string(rc).decode())
    out = np.zeros((n.value, 6), np.int32)
    rc = lib.lwp_enumerate_configs(layer.ctypes.data, int(n_devices), out.ctypes.data, n.value, ctypes.byref(n))
    if rc:
        raise LwpError(rc, "enumerate_configs", lib.lwp_status_string(rc).decode())
    return out


def search_workspace_bytes_ragged(n_nodes, edges, C_node, schedule=SCHEDULE_ROUNDS, undo=UNDO_STORED) -> int:
    lib = load()
    edges = _np_i32(edges, (-1, 2))
    C_node = _np_i32(C_node, (-1,))
    if len(C_node) != n_nodes:
        raise ValueError("C_node must have one entry per node")
    return int(lib.lwp_search_workspace_bytes_ragged(n_nodes, len(edges), edges.ctypes.data, C_node.ctypes.data,
                                                     int(schedule), int(undo)))


_I32 = None      # torch.int32, looked up once (torch is imported on first use only)


def _dev(t, what):
    global _I32
    if _I32 is None:
        import torch
        _I32 = torch.int32
    try:
        if t.is_cuda and t.dtype is _I32 and t.is_contiguous():
            return t.data_ptr()
    except AttributeError:
        pass
    raise TypeError(f"{what} must be a contiguous int32 CUDA tensor")


def eliminate_node_noalloc(A, w, B, out, argmin=None, status=None, stream=None):
    """lwp_eliminate_node_noalloc on the current device: every buffer is the caller's, nothing is allocated.

    A [batch][Ci][Cj], w [batch][Cj], B [batch][Cj][Ck], out (and argmin, optional) [batch][Ci][Ck]:
    contiguous int32 CUDA tensors; status: optional int32 CUDA tensor of one element that receives
    error bits; stream: a torch stream (default: the current one).  Only enqueues."""
    import torch
    lib = load()
    batch, Ci, Cj = A.shape
    Ck = B.shape[2]
    if tuple(B.shape) != (batch, Cj, Ck) or tuple(w.shape) != (batch, Cj) or tuple(out.shape) != (batch, Ci, Ck):
        raise ValueError("shape mismatch between A, w, B and out")
    if argmin is not None and tuple(argmin.shape) != (batch, Ci, Ck):
        raise ValueError("argmin must have the shape of out")
    st = stream if stream is not None else torch.cuda.current_stream()
    rc = lib.lwp_eliminate_node_noalloc(ctypes.c_void_p(st.cuda_stream), batch, Ci, Cj, Ck, _dev(A, "A"), _dev(w, "w"),
                                        _dev(B, "B"), _dev(out, "out"), _dev(argmin, "argmin") if argmin is not None else None,
                                        _dev(status, "status") if status is not None else None)
    if rc:
        raise LwpError(rc, "eliminate_node_noalloc", lib.lwp_status_string(rc).decode())


class SearchPlan:
    """Owns one lwp_search_plan (see Context.search_plan).  Close it before its context."""

    def __init__(self, ctx, n_nodes, edges, C_node, tc, ts, tx, schedule):
        edges = _np_i32(edges, (-1, 2))
        C_node = np.full(n_nodes, int(C_node), np.int32) if np.ndim(C_node) == 0 else _np_i32(C_node, (-1,))
        if len(C_node) != n_nodes:
            raise ValueError("C_node must have one entry per node")
        E = len(edges)
        n_w = int(C_node.astype(np.int64).sum())
        if tc.numel() != n_w or ts.numel() != n_w:
            raise ValueError("t_c / t_s must hold sum(C_node) entries")
        if E and (edges >= 0).all() and (edges < n_nodes).all():
            if tx.numel() != int((C_node[edges[:, 0]].astype(np.int64) * C_node[edges[:, 1]]).sum()):
                raise ValueError("t_x must hold sum(C_src * C_dst) entries")
        self._ctx, self._lib, self.n_nodes = ctx, ctx._lib, n_nodes
        self._tables = (tc, ts, tx)
        h = ctypes.c_void_p()
        rc = self._lib.lwp_search_plan_create(ctx._h, n_nodes, E, edges.ctypes.data, C_node.ctypes.data, _dev(tc, "tc"),
                                              _dev(ts, "ts"), _dev(tx, "tx") if E else None, int(schedule), ctypes.byref(h))
        ctx._check(rc, "search_plan_create")
        self._h = h

    def run(self):
        """Returns (cost, strategy[n_nodes]) for what the tables hold now."""
        cost = ctypes.c_int32(0)
        S, S_ptr = _result_buffer(self.n_nodes)
        rc = self._lib.lwp_search_plan_run(self._h, ctypes.byref(cost), S_ptr)
        self._ctx._check(rc, "search_plan_run")
        return cost.value, S

    def close(self):
        if getattr(self, "_h", None):
            self._lib.lwp_search_plan_destroy(self._h)
            self._h = None

    __del__ = close

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


class Context:
    """Owns one lwp_ctx bound to a device and to torch's current stream on it."""

    def __init__(self, device: int = 0, stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the strategy search has no CPU path")
        self._lib = load()
        self.device = int(device)
        with torch.cuda.device(self.device):
            self._stream = stream if stream is not None else torch.cuda.current_stream()
        h = ctypes.c_void_p()
        rc = self._lib.lwp_create(ctypes.byref(h), self.device, ctypes.c_void_p(self._stream.cuda_stream))
        if rc:
            raise LwpError(rc, "lwp_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.lwp_destroy(self._h)
            self._h = None

    __del__ = close

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _check(self, rc, what):
        if rc:
            raise LwpError(rc, what, self._lib.lwp_last_error(self._h).decode())

    def set_single_launch(self, on=True):
        """Whether very small searches run as one launch of one workgroup (default) or down the general path."""
        self._check(self._lib.lwp_set_option(self._h, 0, 1 if on else 0), "set_option")

    def set_small_product_kernel(self, on=True):
        """Whether node eliminations with little work run on the wavefront-per-tile kernel (default) or on the tiled one."""
        self._check(self._lib.lwp_set_option(self._h, 1, 1 if on else 0), "set_option")

    def synchronize(self):
        self._check(self._lib.lwp_synchronize(self._h), "synchronize")

    # ---- Eq. 2 -------------------------------------------------------------
    def eliminate_node(self, A, w, B, out=None, argmin=None, want_argmin=True, bounds=None):
        """A [batch][Ci][Cj], w [batch][Cj], B [batch][Cj][Ck] -> (out, argmin) [batch][Ci][Ck].

        Only enqueues; synchronize() reports what the kernels found (overflow, broken promise).
        bounds: optional (lo A, hi A, lo w, hi w, lo B, hi B) the caller promises for the values."""
        import torch
        if A.dim() == 2:
            A, w, B = A[None], w[None], B[None]
        batch, Ci, Cj = A.shape
        Ck = B.shape[2]
        if tuple(B.shape) != (batch, Cj, Ck) or tuple(w.shape) != (batch, Cj):
            raise ValueError("shape mismatch between A, w and B")
        if out is None:
            out = torch.empty((batch, Ci, Ck), dtype=torch.int32, device=A.device)
        if argmin is None and want_argmin:
            argmin = torch.empty((batch, Ci, Ck), dtype=torch.int32, device=A.device)
        if bounds is None:
            rc = self._lib.lwp_eliminate_node(self._h, batch, Ci, Cj, Ck, _dev(A, "A"), _dev(w, "w"), _dev(B, "B"),
                                              _dev(out, "out"), _dev(argmin, "argmin") if argmin is not None else None)
        else:
            b = _np_i32(bounds, (6,))
            rc = self._lib.lwp_eliminate_node_bounded(self._h, batch, Ci, Cj, Ck, _dev(A, "A"), _dev(w, "w"), _dev(B, "B"),
                                                      _dev(out, "out"), _dev(argmin, "argmin") if argmin is not None else None,
                                                      b.ctypes.data)
        self._check(rc, "eliminate_node")
        return out, argmin

    # ---- Eq. 3 -------------------------------------------------------------
    def eliminate_edge(self, e1, e2, out=None):
        import torch
        if e1.shape != e2.shape:
            raise ValueError("shape mismatch")
        shp = e1.shape if e1.dim() == 3 else (1,) + tuple(e1.shape)
        if out is None:
            out = torch.empty_like(e1)
        rc = self._lib.lwp_eliminate_edge(self._h, shp[0], shp[1], shp[2], _dev(e1, "e1"), _dev(e2, "e2"), _dev(out, "out"))
        self._check(rc, "eliminate_edge")
        return out

    # ---- Alg. 1 ------------------------------------------------------------
    def search_graph(self, n_nodes, edges, C, tc, ts, tx, schedule=SCHEDULE_ROUNDS, undo=UNDO_STORED):
        """Returns (cost, strategy[n_nodes]) with tables resident on the device."""
        edges = _np_i32(edges, (-1, 2))
        E = len(edges)
        if tuple(tc.shape) != (n_nodes, C) or tuple(ts.shape) != (n_nodes, C):
            raise ValueError("t_c / t_s must be [n_nodes][C]")
        if E and tuple(tx.shape) != (E, C, C):
            raise ValueError("t_x must be [n_edges][C][C]")
        cost = ctypes.c_int32(0)
        S, S_ptr = _result_buffer(n_nodes)
        rc = self._lib.lwp_search_graph_ex(self._h, n_nodes, E, _ptr(edges), C, _dev(tc, "tc"), _dev(ts, "ts"),
                                           _dev(tx, "tx") if E else None, int(schedule), int(undo), ctypes.byref(cost),
                                           S_ptr)
        self._check(rc, "search_graph")
        return cost.value, S

    def search_graph_ragged(self, n_nodes, edges, C_node, tc, ts, tx, schedule=SCHEDULE_ROUNDS, undo=UNDO_STORED):
        """Search with C_node[v] configurations for node v; tc, ts, tx are flat concatenations."""
        edges = _np_i32(edges, (-1, 2))
        C_node = _np_i32(C_node, (-1,))
        E = len(edges)
        if len(C_node) != n_nodes:
            raise ValueError("C_node must have one entry per node")
        n_w = int(C_node.astype(np.int64).sum())
        if tc.dim() != 1 or ts.dim() != 1 or tc.numel() != n_w or ts.numel() != n_w:
            raise ValueError("t_c / t_s must be flat with sum(C_node) entries")
        if E:
            ok = (edges >= 0).all() and (edges < n_nodes).all()
            n_x = int((C_node[edges[:, 0]].astype(np.int64) * C_node[edges[:, 1]]).sum()) if ok else -1
            if ok and (tx.dim() != 1 or tx.numel() != n_x):
                raise ValueError("t_x must be flat with sum(C_src * C_dst) entries")
        cost = ctypes.c_int32(0)
        S, S_ptr = _result_buffer(n_nodes)
        rc = self._lib.lwp_search_graph_ragged(self._h, n_nodes, E, _ptr(edges), _ptr(C_node),
                                               _dev(tc, "tc"), _dev(ts, "ts"), _dev(tx, "tx") if E else None,
                                               int(schedule), int(undo), ctypes.byref(cost), S_ptr)
        self._check(rc, "search_graph_ragged")
        return cost.value, S

    def search_plan(self, n_nodes, edges, C_node, tc, ts, tx, schedule=SCHEDULE_ROUNDS):
        """A search prepared once and run many times: SearchPlan.run() searches the tables' present contents.

        C_node: one count for all nodes or one per node; tc, ts, tx as search_graph / search_graph_ragged
        take them.  The plan keeps the three tensors alive; change their contents in place between runs."""
        return SearchPlan(self, n_nodes, edges, C_node, tc, ts, tx, schedule)

    # ---- Sec. 5.1 ----------------------------------------------------------
    def build_cost_tables(self, layers, edges, configs, machine):
        """layers int32 [L][14], edges [E][2], configs int32 [C][6], machine dict -> (tc, ts, tx) on device."""
        import torch
        layers = _np_i32(layers, (-1, 14))
        edges = _np_i32(edges, (-1, 2))
        configs = _np_i32(configs, (-1, 6))
        m = np.array([machine["n_devices"], machine["flop_per_ns"], machine["byte_per_ns"], machine["invalid_cost"]], np.int32)
        L, E, C = len(layers), len(edges), len(configs)
        dev = torch.device("cuda", self.device)
        tc = torch.empty((L, C), dtype=torch.int32, device=dev)
        ts = torch.empty((L, C), dtype=torch.int32, device=dev)
        tx = torch.empty((E, C, C), dtype=torch.int32, device=dev)
        rc = self._lib.lwp_build_cost_tables(self._h, layers.ctypes.data, L, edges.ctypes.data, E, configs.ctypes.data, C,
                                             m.ctypes.data, _dev(tc, "tc"), _dev(ts, "ts"), _dev(tx, "tx") if E else None)
        self._check(rc, "build_cost_tables")
        return tc, ts, tx

    def build_cost_tables_ragged(self, layers, edges, configs, C_node, machine):
        """Per-layer configuration lists (concatenated in ``configs``, C_node[l] rows for layer l)
        -> flat (tc, ts, tx) on the device, in the layout search_graph_ragged takes."""
        import torch
        layers = _np_i32(layers, (-1, 14))
        edges = _np_i32(edges, (-1, 2))
        configs = _np_i32(configs, (-1, 6))
        C_node = _np_i32(C_node, (-1,))
        L, E = len(layers), len(edges)
        if len(C_node) != L or (C_node < 1).any() or int(C_node.astype(np.int64).sum()) != len(configs):
            raise ValueError("C_node must have one positive entry per layer and sum to the number of rows")
        if E and ((edges < 0).any() or (edges >= L).any()):
            raise ValueError("edge endpoint out of range")
        m = np.array([machine["n_devices"], machine["flop_per_ns"], machine["byte_per_ns"], machine["invalid_cost"]], np.int32)
        rows = int(C_node.astype(np.int64).sum())
        cells = int((C_node[edges[:, 0]].astype(np.int64) * C_node[edges[:, 1]]).sum()) if E else 0
        dev = torch.device("cuda", self.device)
        tc = torch.empty(rows, dtype=torch.int32, device=dev)
        ts = torch.empty(rows, dtype=torch.int32, device=dev)
        tx = torch.empty(max(cells, 1), dtype=torch.int32, device=dev)[:cells]
        rc = self._lib.lwp_build_cost_tables_ragged(self._h, layers.ctypes.data, L, edges.ctypes.data, E,
                                                    configs.ctypes.data, C_node.ctypes.data, m.ctypes.data,
                                                    _dev(tc, "tc"), _dev(ts, "ts"), _dev(tx, "tx") if E else None)
        self._check(rc, "build_cost_tables_ragged")
        return tc, ts, tx

    def build_cost_tables_graph(self, layers, edges, configs, C_node, n_devices, flop_per_ns, invalid_cost, bandwidth,
                                measured_tc=None):
        """As build_cost_tables_ragged on a device graph: bandwidth int32 [n_devices][n_devices] (byte per ns
        from row device to column device); measured_tc (optional, host int32, one entry per configuration
        row) replaces the analytic t_c."""
        import torch
        layers = _np_i32(layers, (-1, 14))
        edges = _np_i32(edges, (-1, 2))
        configs = _np_i32(configs, (-1, 6))
        C_node = _np_i32(C_node, (-1,))
        bandwidth = _np_i32(bandwidth, (int(n_devices), int(n_devices)))
        L, E = len(layers), len(edges)
        if len(C_node) != L or (C_node < 1).any() or int(C_node.astype(np.int64).sum()) != len(configs):
            raise ValueError("C_node must have one positive entry per layer and sum to the number of rows")
        if E and ((edges < 0).any() or (edges >= L).any()):
            raise ValueError("edge endpoint out of range")
        rows = int(C_node.astype(np.int64).sum())
        cells = int((C_node[edges[:, 0]].astype(np.int64) * C_node[edges[:, 1]]).sum()) if E else 0
        mt = None
        if measured_tc is not None:
            mt = _np_i32(measured_tc, (-1,))
            if mt.size != rows:
                raise ValueError("measured_tc must have one entry per configuration row")
        g = DeviceGraph(int(n_devices), int(flop_per_ns), int(invalid_cost), 0, bandwidth.ctypes.data)
        dev = torch.device("cuda", self.device)
        tc = torch.empty(rows, dtype=torch.int32, device=dev)
        ts = torch.empty(rows, dtype=torch.int32, device=dev)
        tx = torch.empty(max(cells, 1), dtype=torch.int32, device=dev)[:cells]
        rc = self._lib.lwp_build_cost_tables_graph(self._h, layers.ctypes.data, L, edges.ctypes.data, E, configs.ctypes.data,
                                                   C_node.ctypes.data, ctypes.byref(g), mt.ctypes.data if mt is not None else None,
                                                   _dev(tc, "tc"), _dev(ts, "ts"), _dev(tx, "tx") if E else None)
        self._check(rc, "build_cost_tables_graph")
        return tc, ts, tx

    # ---- measurement -------------------------------------------------------
    def measure_valu_rate(self):
        """Register-only add + three-way-min loop: dict(lane_ops_per_s, cell_updates_per_s) the device sustains."""
        lane, upd = ctypes.c_double(0), ctypes.c_double(0)
        self._check(self._lib.lwp_measure_valu_rate(self._h, ctypes.byref(lane), ctypes.byref(upd)), "measure_valu_rate")
        return {"lane_ops_per_s": lane.value, "cell_updates_per_s": upd.value}

    def profile_enable(self, on=True):
        self._check(self._lib.lwp_profile_enable(self._h, 1 if on else 0), "profile_enable")

    def profile_reset(self):
        self._check(self._lib.lwp_profile_reset(self._h), "profile_reset")

    def profile_read(self) -> dict:
        p = Profile()
        self._check(self._lib.lwp_profile_read(self._h, ctypes.byref(p)), "profile_read")
        return {f: getattr(p, f) for f, _ in Profile._fields_}
