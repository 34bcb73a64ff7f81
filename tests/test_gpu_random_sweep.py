"""Seeded random sweeps on the GPU against the oracle: launch shapes around the boundaries of the
tile-splitting and kernel-choice rules (Eq. 2), and whole searches on random series-parallel graphs
with a configuration count per node (Alg. 1), down every path the library has (one workgroup or the
general path, wavefront-per-tile or tiled kernel, stored or recomputed argmin)."""
import numpy as np
import pytest

import oracle
from paper_1802_04924_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import torch
    from paper_1802_04924_amd import Context
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    with Context(0) as c:
        yield c


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("seed", [11, 12])
def test_random_launch_shapes(ctx, seed):
    rng = np.random.default_rng(seed)
    for case in range(500):
        Ci, Ck = int(rng.integers(1, 700)), int(rng.integers(1, 700))
        Cj = int(rng.choice([rng.integers(1, 64), rng.integers(64, 400), rng.integers(400, 1200)]))
        tiles_per = -(-Ci // 64) * -(-Ck // 64)
        target = int(rng.choice([rng.integers(1, 64), rng.integers(64, 300), rng.integers(300, 1400)]))
        batch = max(1, min(target // tiles_per, int(4e8 // (Ci * Cj * Ck)) or 1))
        hi = int(rng.choice([2, 1000, 1 << 20, 1 << 27]))
        lo = int(rng.choice([0, -hi]))
        A = rng.integers(lo, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
        w = rng.integers(0, hi, size=(batch, Cj), endpoint=True, dtype=np.int32)
        B = rng.integers(lo, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
        dA, dw, dB = dev(A), dev(w), dev(B)
        picks = sorted({0, batch - 1, int(rng.integers(0, batch))})
        ref = {b: oracle.minplus_argmin(A[b], w[b], B[b]) for b in picks}
        for wave in (True, False):
            ctx.set_small_product_kernel(wave)
            for bounds in (None, (lo, hi, 0, hi, lo, hi)):
                out, arg = ctx.eliminate_node(dA, dw, dB, bounds=bounds)
                ctx.synchronize()
                out, arg = out.cpu().numpy(), arg.cpu().numpy()
                for b in picks:
                    assert np.array_equal(out[b], ref[b][0]) and np.array_equal(arg[b], ref[b][1]), \
                        (case, batch, Ci, Cj, Ck, lo, hi, wave, bounds is not None, b)
    ctx.set_small_product_kernel(True)


@pytest.mark.parametrize("seed0", [5, 6])
def test_random_searches(ctx, seed0):
    from paper_1802_04924_amd import plan_graph
    rng = np.random.default_rng(seed0)
    for case in range(1500):
        seed = int(rng.integers(0, 1 << 30))
        n, edges = wl.series_parallel_edges(int(rng.integers(2, 60)), seed, p_branch=float(rng.choice([0.0, 0.05, 0.1])))
        c_max = int(rng.choice([2, 5, 12, 24, 40, 90, 170]))
        Cn = wl.ragged_counts(n, seed + 1, 1, c_max)
        k = plan_graph(n, edges)["n_residual_nodes"]
        if k > 2 and float(c_max) ** k > (1 << 26):
            Cn = wl.ragged_counts(n, seed + 1, 1, 3)     # keep the residual enumeration small on both sides
        hi = int(rng.choice([2, 1000, 1 << 20]))
        tc, ts, tx = wl.ragged_tables(n, edges, Cn, seed + 2, 0, hi)
        d = (dev(tc), dev(ts), dev(tx))
        for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
            ref = oracle.search_ragged(n, edges, Cn, tc, ts, tx, schedule)
            for single in (True, False):
                ctx.set_single_launch(single)
                for wave in (True, False):
                    ctx.set_small_product_kernel(wave)
                    for undo in (0, 1):
                        cost, S = ctx.search_graph_ragged(n, edges, Cn, *d, schedule, undo)
                        assert cost == ref["cost"] and np.array_equal(S, ref["strategy"]), \
                            (case, seed, c_max, hi, schedule, single, wave, undo)
    ctx.set_single_launch(True)
    ctx.set_small_product_kernel(True)


def test_random_searches_with_one_count_for_all_nodes(ctx):
    # the uniform entry point (one C for every node) on the same kind of graphs
    from paper_1802_04924_amd import plan_graph
    rng = np.random.default_rng(7)
    for case in range(600):
        seed = int(rng.integers(0, 1 << 30))
        n_ops = int(rng.integers(2, 50))
        C = int(rng.choice([1, 2, 3, 7, 16, 33, 64, 100]))
        n, edges = wl.series_parallel_edges(n_ops, seed, p_branch=float(rng.choice([0.0, 0.1])))
        k = plan_graph(n, edges)["n_residual_nodes"]
        if k > 2 and float(C) ** k > (1 << 26):
            C = 3
        hi = int(rng.choice([1, 1000, 1 << 22]))
        tc, ts, tx = wl.random_tables(n, edges, C, seed + 3, (0, hi), (0, hi), (0, hi))
        d = (dev(tc), dev(ts), dev(tx))
        for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
            ref = oracle.search(n, edges, C, tc, ts, tx, schedule)
            for single in (True, False):
                ctx.set_single_launch(single)
                for undo in (0, 1):
                    cost, S = ctx.search_graph(n, edges, C, *d, schedule, undo)
                    assert cost == ref["cost"] and np.array_equal(S, ref["strategy"]), (case, seed, C, hi, schedule, single, undo)
    ctx.set_single_launch(True)


def test_random_cost_tables(ctx):
    # Sec. 5.1 on random small networks: chains of convolution / pooling / fully connected layers with
    # consistent shapes (odd extents, strides, paddings), per-layer configuration lists for 2 to 16 devices
    from paper_1802_04924_amd import enumerate_configs
    rng = np.random.default_rng(51)
    for case in range(150):
        N = int(rng.integers(1, 9))
        C, H, W = int(rng.integers(1, 9)), int(rng.integers(4, 30)), int(rng.integers(4, 30))
        layers = []
        fc_seen = False
        for _ in range(int(rng.integers(2, 6))):
            kind = wl.KIND_FC if fc_seen else int(rng.choice([wl.KIND_CONV, wl.KIND_CONV, wl.KIND_POOL, wl.KIND_FC]))
            if kind == wl.KIND_FC:
                Co = int(rng.integers(1, 12))
                layers.append((kind, N, C, H, W, Co, 1, 1, H, W, 1, 1, 0, 0))
                C, H, W, fc_seen = Co, 1, 1, True
                continue
            kh, kw = int(rng.integers(1, min(5, H) + 1)), int(rng.integers(1, min(5, W) + 1))
            sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
            ph, pw = (int(rng.integers(0, kh // 2 + 1)), int(rng.integers(0, kw // 2 + 1))) if kind == wl.KIND_CONV else (0, 0)
            Ho, Wo = (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1
            Co = int(rng.integers(1, 12)) if kind == wl.KIND_CONV else C
            layers.append((kind, N, C, H, W, Co, Ho, Wo, kh, kw, sh, sw, ph, pw))
            C, H, W = Co, Ho, Wo
        layers = np.asarray(layers, np.int32)
        edges = wl.chain_edges(len(layers))
        n_dev = int(rng.choice([2, 3, 4, 6, 8, 12, 16]))
        m = {"n_devices": n_dev, "flop_per_ns": int(rng.integers(1, 2000)), "byte_per_ns": int(rng.integers(1, 50)),
             "invalid_cost": 1 << 27}
        lists = [enumerate_configs(l, n_dev) for l in layers]
        configs, Cn = np.concatenate(lists), np.array([len(x) for x in lists], np.int32)
        tc, ts, tx = ctx.build_cost_tables_ragged(layers, edges, configs, Cn, m)
        rtc, rts, rtx = oracle.build_cost_tables_ragged(layers, edges, configs, Cn, m)
        assert np.array_equal(tc.cpu().numpy(), rtc), (case, "tc")
        assert np.array_equal(ts.cpu().numpy(), rts), (case, "ts")
        assert np.array_equal(tx.cpu().numpy(), rtx), (case, "tx")
        ref = oracle.search_ragged(len(layers), edges, Cn, rtc, rts, rtx)
        cost, S = ctx.search_graph_ragged(len(layers), edges, Cn, tc, ts, tx)
        assert cost == ref["cost"] and np.array_equal(S, ref["strategy"]), case
        # the same network on a device graph (Sec. 4): a bandwidth per ordered pair of devices, and every
        # third time t_c handed in instead of computed
        bw = rng.choice([1, 2, 4, 5, 8, 10, 16, 20, 25, 40, 50], size=(n_dev, n_dev)).astype(np.int32)
        mt = rng.integers(1, 1 << 20, size=int(Cn.sum()), dtype=np.int32) if case % 3 == 0 else None
        g = ctx.build_cost_tables_graph(layers, edges, configs, Cn, n_dev, m["flop_per_ns"], m["invalid_cost"], bw, mt)
        r = oracle.build_cost_tables_graph(layers, edges, configs, Cn, n_dev, m["flop_per_ns"], m["invalid_cost"], bw, mt)
        for name, a, b in zip(("tc", "ts", "tx"), g, r):
            assert np.array_equal(a.cpu().numpy(), b), (case, "graph", name)
