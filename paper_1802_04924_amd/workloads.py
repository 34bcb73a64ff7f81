"""Seeded synthetic inputs for the strategy search (graphs, cost tables, layer
and configuration descriptors).

This module only *draws inputs*.  It contains none of the method's arithmetic
(no cost formula, no elimination, no min-plus); both the CPU oracle's tests and
the GPU library's tests feed on the arrays produced here so that the two sides
see identical bits.

All random tables come from ``numpy.random.Generator(PCG64(seed))`` with
``integers(lo, hi, endpoint=True)`` drawn in the fixed order t_c, t_s, t_x.
"""
from __future__ import annotations

import numpy as np

# Schedules understood by both the oracle and the GPU library.
SCHEDULE_ROUNDS = 0      # batched rounds of independent eliminations
SCHEDULE_LEFT_FOLD = 1   # one node elimination per round, lowest eligible id
SCHEDULE_NONE = 2        # no elimination: every strategy of the original graph is enumerated (the paper's baseline)

# Layer kinds for the analytic cost model inputs.
KIND_CONV, KIND_POOL, KIND_FC = 0, 1, 2

LAYER_FIELDS = ("kind", "N", "Cin", "Hin", "Win", "Cout", "Hout", "Wout",
                "kh", "kw", "sh", "sw", "ph", "pw")
CONFIG_FIELDS = ("n", "h", "w", "c", "dev_offset", "pad")


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def chain_edges(n_nodes: int) -> np.ndarray:
    """Edge list (l, l+1) of a chain of ``n_nodes`` layers."""
    e = np.stack([np.arange(n_nodes - 1), np.arange(1, n_nodes)], axis=1)
    return np.ascontiguousarray(e, dtype=np.int32).reshape(-1, 2)


def random_tables(n_nodes, edges, C, seed, tc_range, ts_range, tx_range):
    """Uniform int32 tables t_c[N][C], t_s[N][C], t_x[E][C][C]."""
    rng = _rng(seed)
    E = len(edges)
    tc = rng.integers(tc_range[0], tc_range[1], size=(n_nodes, C), endpoint=True, dtype=np.int32)
    ts = rng.integers(ts_range[0], ts_range[1], size=(n_nodes, C), endpoint=True, dtype=np.int32)
    tx = rng.integers(tx_range[0], tx_range[1], size=(E, C, C), endpoint=True, dtype=np.int32)
    return tc, ts, tx


def ragged_tables(n_nodes, edges, Cn, seed, lo=0, hi=1000):
    """Tables for per-node configuration counts Cn: t_c and t_s are the rows of all nodes one after
    another, t_x the tables [Cn[src]][Cn[dst]] of all edges one after another (flat int32 arrays)."""
    rng = _rng(seed)
    Cn = np.asarray(Cn, dtype=np.int32)
    total = int(Cn.sum())
    cells = int(sum(int(Cn[i]) * int(Cn[j]) for i, j in np.asarray(edges).reshape(-1, 2)))
    tc = rng.integers(lo, hi, size=total, endpoint=True, dtype=np.int32)
    ts = rng.integers(lo, hi, size=total, endpoint=True, dtype=np.int32)
    tx = rng.integers(lo, hi, size=cells, endpoint=True, dtype=np.int32)
    return tc, ts, tx


def ragged_counts(n_nodes, seed, c_min, c_max):
    """Seeded per-node configuration counts in [c_min, c_max]."""
    return _rng(seed).integers(c_min, c_max, size=n_nodes, endpoint=True, dtype=np.int32)


def _problem(name, n_nodes, edges, C, tc, ts, tx, schedule):
    return {"name": name, "n_nodes": int(n_nodes), "edges": np.ascontiguousarray(edges, dtype=np.int32),
            "C": int(C), "tc": tc, "ts": ts, "tx": tx, "schedule": schedule}


def chain_problem(n_layers, C, seed, tc_range=(1, 1000), ts_range=(1, 1000), tx_range=(0, 1000),
                  schedule=SCHEDULE_ROUNDS, name="chain"):
    edges = chain_edges(n_layers)
    tc, ts, tx = random_tables(n_layers, edges, C, seed, tc_range, ts_range, tx_range)
    return _problem(name, n_layers, edges, C, tc, ts, tx, schedule)


def config0():
    """Chain of 6 layers, 16 configurations each, seed 0 (LeNet-5-sized, cf. Table 3)."""
    return chain_problem(6, 16, 0, name="cfg0_chain6_C16")


def forkjoin_edges(n_modules: int, seed: int):
    """Inception-shaped DAG: ``n_modules`` fork/join modules of 12 nodes.

    Module m has a fork node F, four branches and a join node J.  Even modules
    use branch lengths (3,3,2,2), odd modules (3,3,3,1), each in a seeded
    permutation, so every module has 10 branch nodes with 1-3 nodes per branch.
    Node ids are topological: F, then the branches one after another, then J.
    Edges: along every branch F->b1->...->bk->J, the last edge of every branch
    twice (a parallel pair), and J_m -> F_{m+1}.
    """
    rng = _rng(seed)
    edges = []
    for m in range(n_modules):
        base = 12 * m
        lens = np.array([3, 3, 2, 2] if m % 2 == 0 else [3, 3, 3, 1])
        lens = lens[rng.permutation(4)]
        F, J = base, base + 11
        nid = base + 1
        for L in lens:
            prev = F
            for _ in range(int(L)):
                edges.append((prev, nid))
                prev = nid
                nid += 1
            edges.append((prev, J))
            edges.append((prev, J))          # duplicated tail edge
        assert nid == J
        if m + 1 < n_modules:
            edges.append((J, base + 12))
    return 12 * n_modules, np.asarray(edges, dtype=np.int32).reshape(-1, 2)


def forkjoin_problem(n_modules, C, seed, lo=1, hi=100000, schedule=SCHEDULE_ROUNDS, name="forkjoin"):
    n_nodes, edges = forkjoin_edges(n_modules, seed)
    # the graph draws come first from their own generator; tables use seed too but a fresh stream
    tc, ts, tx = random_tables(n_nodes, edges, C, seed + 1000003, (lo, hi), (lo, hi), (lo, hi))
    return _problem(name, n_nodes, edges, C, tc, ts, tx, schedule)


def resnet_edges(blocks_per_stage=(3, 4, 6, 3), bottleneck: bool = False):
    """ResNet-shaped DAG: a stem (convolution, pooling), stages of residual blocks, pooling and a
    fully connected layer.  A block is 2 (``bottleneck``: 3) convolutions followed by an element-wise
    addition that also receives the block's input; the first block of every stage after the first
    has a projection convolution on the skip path.  Node ids are topological.  The default is
    ResNet-34's block counts (55 nodes); (3, 4, 6, 3) with bottlenecks is ResNet-50-shaped."""
    edges = []
    nid = 2
    edges.append((0, 1))                 # stem convolution -> pooling
    prev = 1
    for stage, n_blocks in enumerate(blocks_per_stage):
        for b in range(n_blocks):
            x = prev
            for _ in range(3 if bottleneck else 2):
                edges.append((prev, nid))
                prev = nid
                nid += 1
            if b == 0 and stage > 0:     # projection on the skip path
                edges.append((x, nid))
                skip = nid
                nid += 1
            else:
                skip = x
            add = nid
            nid += 1
            edges.append((prev, add))
            edges.append((skip, add))
            prev = add
    edges.append((prev, nid))            # global pooling
    edges.append((nid, nid + 1))         # fully connected
    return nid + 2, np.asarray(edges, dtype=np.int32).reshape(-1, 2)


def resnet_problem(C, seed, blocks_per_stage=(3, 4, 6, 3), bottleneck=False, lo=1, hi=100000,
                   schedule=SCHEDULE_ROUNDS):
    n_nodes, edges = resnet_edges(blocks_per_stage, bottleneck)
    tc, ts, tx = random_tables(n_nodes, edges, C, seed, (lo, hi), (lo, hi), (lo, hi))
    return _problem(f"resnet{n_nodes}_C{C}", n_nodes, edges, C, tc, ts, tx, schedule)


def config2(C: int = 512, n_modules: int = 10):
    """Inception-shaped DAG, 120 nodes / 189 edges at the default size."""
    return forkjoin_problem(n_modules, C, 2, name=f"cfg2_forkjoin{n_modules}_C{C}")


def series_parallel_edges(n_ops: int, seed: int, p_parallel: float = 0.3, p_branch: float = 0.15,
                          max_branches: int = 2):
    """Random two-terminal DAG grown from one edge by series splits (an edge gets a new node in
    the middle), parallel duplications (an edge is doubled) and, with probability ``p_branch``,
    dangling branches (a new sink hanging off an existing node, which makes the residual graph
    larger than two nodes; at most ``max_branches`` of them).  Node ids are assigned in creation
    order, so they are NOT topological.
    """
    rng = _rng(seed)
    edges = [(0, 1)]
    n = 2
    branches = 0
    for _ in range(n_ops):
        r = rng.random()
        e = int(rng.integers(0, len(edges)))
        if r < p_branch and branches < max_branches:
            branches += 1
            edges.append((edges[e][int(rng.integers(0, 2))], n))
            n += 1
        elif r < p_branch + p_parallel:
            edges.append(edges[e])
        else:
            a, b = edges[e]
            edges[e] = (a, n)
            edges.append((n, b))
            n += 1
    order = rng.permutation(len(edges))
    return n, np.asarray([edges[i] for i in order], dtype=np.int32).reshape(-1, 2)


def series_parallel_problem(n_ops, C, seed, hi=1000, schedule=SCHEDULE_ROUNDS, p_branch=0.0):
    n_nodes, edges = series_parallel_edges(n_ops, seed, p_branch=p_branch)
    tc, ts, tx = random_tables(n_nodes, edges, C, seed + 77, (0, hi), (0, hi), (0, hi))
    return _problem(f"sp{n_ops}_C{C}", n_nodes, edges, C, tc, ts, tx, schedule)


def batched_products(batch, Ci, Cj, Ck, seed, hi=1 << 20):
    """Independent (A, w, B) triples for the isolated node-elimination kernel."""
    rng = _rng(seed)
    A = rng.integers(0, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
    w = rng.integers(0, hi, size=(batch, Cj), endpoint=True, dtype=np.int32)
    B = rng.integers(0, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
    return A, w, B


def config3(batch: int = 4096, C: int = 256):
    return batched_products(batch, C, C, C, 3)


def config4(n_layers: int = 64, C: int = 4096):
    """Long chain with many configurations per layer; left-fold schedule."""
    hi = 1 << 20
    return chain_problem(n_layers, C, 4, (0, hi), (0, hi), (0, hi),
                         schedule=SCHEDULE_LEFT_FOLD, name=f"cfg4_chain{n_layers}_C{C}")


# ---------------------------------------------------------------------------
# Inputs of the analytic cost model (config 1): layer shapes, configuration
# enumeration, machine constants.  Pure descriptors; the formulas live elsewhere.
# ---------------------------------------------------------------------------

def alexnet_layers(batch: int = 256) -> np.ndarray:
    """11-layer AlexNet-shaped chain as an int32 array [11][14] (LAYER_FIELDS).

    Shapes agree with the two AlexNet rows the paper lists (conv2: 64->192
    channels at 27x27 with a 5x5 kernel; conv5: 256->256 at 13x13 with 3x3).
    """
    def conv(cin, hin, cout, k, s, p):
        hout = (hin + 2 * p - k) // s + 1
        return (KIND_CONV, batch, cin, hin, hin, cout, hout, hout, k, k, s, s, p, p)

    def pool(c, hin, k, s):
        hout = (hin - k) // s + 1
        return (KIND_POOL, batch, c, hin, hin, c, hout, hout, k, k, s, s, 0, 0)

    def fc(cin, hin, cout):
        return (KIND_FC, batch, cin, hin, hin, cout, 1, 1, hin, hin, 1, 1, 0, 0)

    layers = [
        conv(3, 224, 64, 11, 4, 2),    # conv1 -> 55
        pool(64, 55, 3, 2),            # pool1 -> 27
        conv(64, 27, 192, 5, 1, 2),    # conv2 -> 27
        pool(192, 27, 3, 2),           # pool2 -> 13
        conv(192, 13, 384, 3, 1, 1),   # conv3
        conv(384, 13, 256, 3, 1, 1),   # conv4
        conv(256, 13, 256, 3, 1, 1),   # conv5
        pool(256, 13, 3, 2),           # pool3 -> 6
        fc(256, 6, 4096),              # fc6
        fc(4096, 1, 4096),             # fc7
        fc(4096, 1, 1000),             # fc8
    ]
    return np.asarray(layers, dtype=np.int32)


def vgg16_layers(batch: int = 64) -> np.ndarray:
    """21-layer VGG-16-shaped chain (13 3x3 convolutions, 5 poolings, 3 fully connected layers,
    224x224 input), the third network of the paper's search-time table."""
    def conv(cin, hin, cout):
        return (KIND_CONV, batch, cin, hin, hin, cout, hin, hin, 3, 3, 1, 1, 1, 1)

    def pool(c, hin):
        return (KIND_POOL, batch, c, hin, hin, c, hin // 2, hin // 2, 2, 2, 2, 2, 0, 0)

    def fc(cin, hin, cout):
        return (KIND_FC, batch, cin, hin, hin, cout, 1, 1, hin, hin, 1, 1, 0, 0)

    layers, c, h = [], 3, 224
    for width, reps in ((64, 2), (128, 2), (256, 3), (512, 3), (512, 3)):
        for _ in range(reps):
            layers.append(conv(c, h, width))
            c = width
        layers.append(pool(c, h))
        h //= 2
    layers += [fc(512, 7, 4096), fc(4096, 1, 4096), fc(4096, 1, 1000)]
    return np.asarray(layers, dtype=np.int32)


def vgg16_problem(batch: int = 64):
    """Descriptors of the VGG-16-shaped chain (tables come from the cost model)."""
    layers = vgg16_layers(batch)
    return {"name": "vgg16_C256", "layers": layers, "edges": chain_edges(len(layers)),
            "configs": config_table(16, 256), "machine": machine(), "C": 256,
            "n_nodes": len(layers), "schedule": SCHEDULE_ROUNDS}


def config_table(n_devices: int = 16, n_rows: int = 256) -> np.ndarray:
    """Configuration enumeration as int32 [n_rows][6] (CONFIG_FIELDS).

    Rows: every (n, h, w, c) of power-of-two degrees whose product d divides
    into ``n_devices`` (d <= n_devices), each with the device-block offsets
    0, d, 2d, ... ; sorted lexicographically by (n, h, w, c, offset); then
    padding rows (all zeros, ``n == 0`` marks padding) up to ``n_rows``.
    """
    pows = [1 << i for i in range(n_devices.bit_length()) if (1 << i) <= n_devices]
    rows = []
    for n in pows:
        for h in pows:
            for w in pows:
                for c in pows:
                    d = n * h * w * c
                    if d > n_devices:
                        continue
                    for off in range(0, n_devices - d + 1, d):
                        rows.append((n, h, w, c, off, 0))
    rows.sort()
    if len(rows) > n_rows:
        raise ValueError("enumeration larger than the requested table")
    rows += [(0, 0, 0, 0, 0, 0)] * (n_rows - len(rows))
    return np.asarray(rows, dtype=np.int32)


def machine(n_devices: int = 16, flop_per_ns: int = 10_000, byte_per_ns: int = 10,
            invalid_cost: int = 1 << 28):
    """Machine constants: 10 TFLOP/s per device, 10 GB/s links, 2^28 ns sentinel."""
    return {"n_devices": n_devices, "flop_per_ns": flop_per_ns, "byte_per_ns": byte_per_ns,
            "invalid_cost": invalid_cost}


def config1(batch: int = 256):
    """Descriptors for the AlexNet-shaped chain whose tables the cost model builds."""
    layers = alexnet_layers(batch)
    return {"name": "cfg1_alexnet11_C256", "layers": layers, "edges": chain_edges(len(layers)),
            "configs": config_table(16, 256), "machine": machine(), "C": 256,
            "n_nodes": len(layers), "schedule": SCHEDULE_ROUNDS}
