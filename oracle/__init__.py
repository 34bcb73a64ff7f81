"""CPU oracle (TEST INFRASTRUCTURE, not the product).

Thin ctypes wrappers around ``lwp_oracle.c`` (plain C, compiled with gcc) plus
``brute.py`` (exhaustive enumeration of Eq. 1).  Nothing in the GPU package
imports this; only tests, the smoke check and the benchmark's cpu_baseline leg do.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_HERE, "lwp_oracle.c"), os.path.join(_HERE, "cost_model_oracle.c")]
_LIB_PATH = os.path.join(_HERE, "liblwp_oracle.so")
_lib = None

OK, E_INVAL, E_NOT_REDUCIBLE, E_OVERFLOW, E_NOMEM = 0, -1, -3, -4, -5
SCHEDULE_ROUNDS, SCHEDULE_LEFT_FOLD, SCHEDULE_NONE = 0, 1, 2

_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: oracle status {code}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the oracle's C sources into a shared library next to them."""
    srcs = [s for s in _SRC if os.path.exists(s)]
    if not force and os.path.exists(_LIB_PATH) and all(
            os.path.getmtime(_LIB_PATH) >= os.path.getmtime(s) for s in srcs):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", _LIB_PATH] + srcs
    subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB_PATH)
    return _lib


def _p(a):
    return a.ctypes.data_as(_i32p)


def _c(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def omp_threads() -> int:
    """Threads the C loops use (OpenMP default unless OMP_NUM_THREADS is set)."""
    n = os.environ.get("OMP_NUM_THREADS")
    return int(n) if n else (os.cpu_count() or 1)


def strategy_cost(n_nodes, edges, C, tc, ts, tx, S) -> int:
    """Eq. 1 for a complete strategy S, from the original tables."""
    lib = _load()
    edges, tc, ts, tx, S = _c(edges).reshape(-1, 2), _c(tc), _c(ts), _c(tx), _c(S)
    out = ctypes.c_int64(0)
    rc = lib.orc_strategy_cost(n_nodes, len(edges), _p(edges), C, _p(tc), _p(ts), _p(tx), _p(S),
                               ctypes.byref(out))
    if rc:
        raise OracleError(rc, "strategy_cost")
    return out.value


def minplus_argmin(A, w, B):
    """Eq. 2: returns (out[Ci][Ck], arg[Ci][Ck]) for A[Ci][Cj], w[Cj], B[Cj][Ck]."""
    lib = _load()
    A, w, B = _c(A), _c(w), _c(B)
    Ci, Cj = A.shape
    Ck = B.shape[1]
    assert B.shape[0] == Cj and w.shape == (Cj,)
    out = np.empty((Ci, Ck), np.int32)
    arg = np.empty((Ci, Ck), np.int32)
    rc = lib.orc_minplus_argmin(Ci, Cj, Ck, _p(A), _p(w), _p(B), _p(out), _p(arg))
    if rc:
        raise OracleError(rc, "minplus_argmin")
    return out, arg


def edge_sum(e1, e2):
    """Eq. 3."""
    lib = _load()
    e1, e2 = _c(e1), _c(e2)
    out = np.empty_like(e1)
    rc = lib.orc_edge_sum(e1.shape[0], e1.shape[1], _p(e1), _p(e2), _p(out))
    if rc:
        raise OracleError(rc, "edge_sum")
    return out


def final_pair(wi, T, wk):
    """Residual two-node graph: (cost, a, b) with the lowest flat index among equals."""
    lib = _load()
    wi, T, wk = _c(wi), _c(T), _c(wk)
    cost = ctypes.c_int64(0)
    a, b = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib.orc_final_pair(T.shape[0], T.shape[1], _p(wi), _p(T), _p(wk), ctypes.byref(cost),
                            ctypes.byref(a), ctypes.byref(b))
    if rc:
        raise OracleError(rc, "final_pair")
    return cost.value, a.value, b.value


STEP_DTYPE = np.dtype([("kind", "<i4"), ("j", "<i4"), ("i", "<i4"), ("k", "<i4"),
                       ("e1", "<i4"), ("e2", "<i4"), ("round", "<i4")])


def search(n_nodes, edges, C, tc, ts, tx, schedule=SCHEDULE_ROUNDS):
    """Alg. 1.  Returns dict(cost, strategy, steps, n_rounds)."""
    lib = _load()
    edges, tc, ts, tx = _c(edges).reshape(-1, 2), _c(tc), _c(ts), _c(tx)
    E = len(edges)
    assert tc.shape == (n_nodes, C) and ts.shape == (n_nodes, C) and tx.shape == (E, C, C)
    S = np.empty(n_nodes, np.int32)
    steps = np.zeros(max(E, 1), STEP_DTYPE)
    cost = ctypes.c_int64(0)
    n_steps, n_rounds = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib.orc_search(n_nodes, E, _p(edges), C, _p(tc), _p(ts), _p(tx), int(schedule),
                        ctypes.byref(cost), _p(S), steps.ctypes.data_as(ctypes.c_void_p),
                        ctypes.byref(n_steps), ctypes.byref(n_rounds))
    if rc:
        raise OracleError(rc, "search")
    return {"cost": cost.value, "strategy": S, "steps": steps[:n_steps.value],
            "n_rounds": n_rounds.value}


def _ragged_args(n_nodes, edges, Cn, tc, ts, tx):
    edges, Cn = _c(edges).reshape(-1, 2), _c(Cn).reshape(-1)
    tc, ts, tx = _c(tc).reshape(-1), _c(ts).reshape(-1), _c(tx).reshape(-1)
    assert len(Cn) == n_nodes and tc.size == int(Cn.sum()) and ts.size == tc.size
    assert tx.size == int(sum(int(Cn[i]) * int(Cn[j]) for i, j in edges))
    return edges, Cn, tc, ts, tx


def strategy_cost_ragged(n_nodes, edges, Cn, tc, ts, tx, S) -> int:
    """Eq. 1 with Cn[l] configurations for node l; tc, ts, tx are the concatenated rows / tables."""
    lib = _load()
    edges, Cn, tc, ts, tx = _ragged_args(n_nodes, edges, Cn, tc, ts, tx)
    S = _c(S)
    out = ctypes.c_int64(0)
    rc = lib.orc_strategy_cost_ragged(n_nodes, len(edges), _p(edges), _p(Cn), _p(tc), _p(ts), _p(tx), _p(S), ctypes.byref(out))
    if rc:
        raise OracleError(rc, "strategy_cost_ragged")
    return out.value


def search_ragged(n_nodes, edges, Cn, tc, ts, tx, schedule=SCHEDULE_ROUNDS):
    """Alg. 1 with per-node configuration counts.  Returns dict(cost, strategy, steps, n_rounds)."""
    lib = _load()
    edges, Cn, tc, ts, tx = _ragged_args(n_nodes, edges, Cn, tc, ts, tx)
    E = len(edges)
    S = np.empty(n_nodes, np.int32)
    steps = np.zeros(max(E, 1), STEP_DTYPE)
    cost = ctypes.c_int64(0)
    n_steps, n_rounds = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib.orc_search_ragged(n_nodes, E, _p(edges), _p(Cn), _p(tc), _p(ts), _p(tx), int(schedule),
                               ctypes.byref(cost), _p(S), steps.ctypes.data_as(ctypes.c_void_p),
                               ctypes.byref(n_steps), ctypes.byref(n_rounds))
    if rc:
        raise OracleError(rc, "search_ragged")
    return {"cost": cost.value, "strategy": S, "steps": steps[:n_steps.value], "n_rounds": n_rounds.value}


def _machine(machine):
    return np.array([machine["n_devices"], machine["flop_per_ns"], machine["byte_per_ns"],
                     machine["invalid_cost"]], np.int32)


def enumerate_configs(layer, n_devices):
    """Configurations of one layer (Sec. 4 / Table 1, reading in cost_model_oracle.c): int32 [C][6]."""
    lib = _load()
    layer = _c(layer).reshape(14)
    n = lib.orc_enumerate_configs(_p(layer), int(n_devices), None, 0)
    out = np.zeros((n, 6), np.int32)
    assert lib.orc_enumerate_configs(_p(layer), int(n_devices), _p(out), n) == n
    return out


def build_cost_tables_ragged(layers, edges, configs, Cn, machine):
    """Cost tables with a configuration list per layer (lists concatenated in ``configs``).

    Returns flat (tc, ts, tx) in the layout search_ragged takes."""
    lib = _load()
    layers = _c(layers).reshape(-1, 14)
    edges = _c(edges).reshape(-1, 2)
    configs = _c(configs).reshape(-1, 6)
    Cn = _c(Cn).reshape(-1)
    if len(Cn) != len(layers) or int(Cn.sum()) != len(configs):
        raise ValueError("Cn must have one entry per layer and sum to the number of rows")
    m = _machine(machine)
    total = int(Cn.astype(np.int64).sum())
    cells = int(sum(int(Cn[i]) * int(Cn[j]) for i, j in edges))
    tc, ts, tx = np.empty(total, np.int32), np.empty(total, np.int32), np.empty(cells, np.int32)
    rc = lib.orc_build_cost_tables_ragged(_p(layers), len(layers), _p(edges), len(edges), _p(configs), _p(Cn),
                                          _p(m), _p(tc), _p(ts), _p(tx))
    if rc:
        raise OracleError(rc, "build_cost_tables_ragged")
    return tc, ts, tx


def build_cost_tables(layers, edges, configs, machine):
    """Analytic cost model of Sec. 5.1 (readings in cost_model_oracle.c): returns (tc, ts, tx)."""
    lib = _load()
    layers = _c(layers).reshape(-1, 14)
    edges = _c(edges).reshape(-1, 2)
    configs = _c(configs).reshape(-1, 6)
    m = np.array([machine["n_devices"], machine["flop_per_ns"], machine["byte_per_ns"],
                  machine["invalid_cost"]], np.int32)
    L, E, C = len(layers), len(edges), len(configs)
    tc = np.empty((L, C), np.int32)
    ts = np.empty((L, C), np.int32)
    tx = np.empty((E, C, C), np.int32)
    rc = lib.orc_build_cost_tables(_p(layers), L, _p(edges), E, _p(configs), C, _p(m), _p(tc), _p(ts), _p(tx))
    if rc:
        raise OracleError(rc, "build_cost_tables")
    return tc, ts, tx


def build_cost_tables_graph(layers, edges, configs, Cn, n_devices, flop_per_ns, invalid_cost, bandwidth, measured_tc=None):
    """Cost tables on a device graph (Sec. 4: bandwidth[u][v] = b(d_u, d_v) in bytes per ns) with per-layer
    configuration lists; measured_tc (optional, layout of tc) replaces the analytic t_c (Sec. 5.1).

    Returns flat (tc, ts, tx) in the layout search_ragged takes."""
    lib = _load()
    layers = _c(layers).reshape(-1, 14)
    edges = _c(edges).reshape(-1, 2)
    configs = _c(configs).reshape(-1, 6)
    Cn = _c(Cn).reshape(-1)
    bandwidth = _c(bandwidth).reshape(n_devices, n_devices)
    if len(Cn) != len(layers) or int(Cn.sum()) != len(configs):
        raise ValueError("Cn must have one entry per layer and sum to the number of rows")
    total = int(Cn.astype(np.int64).sum())
    cells = int(sum(int(Cn[i]) * int(Cn[j]) for i, j in edges))
    tc, ts, tx = np.empty(total, np.int32), np.empty(total, np.int32), np.empty(max(cells, 1), np.int32)
    mt = None
    if measured_tc is not None:
        mt = _c(measured_tc).reshape(-1)
        if mt.size != total:
            raise ValueError("measured_tc must have one entry per configuration row")
    rc = lib.orc_build_cost_tables_graph(_p(layers), len(layers), _p(edges), len(edges), _p(configs), _p(Cn),
                                         int(n_devices), int(flop_per_ns), int(invalid_cost), _p(bandwidth),
                                         _p(mt) if mt is not None else None, _p(tc), _p(ts), _p(tx))
    if rc:
        raise OracleError(rc, "build_cost_tables_graph")
    return tc, ts, tx[:cells]
