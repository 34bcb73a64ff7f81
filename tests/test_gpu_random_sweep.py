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
