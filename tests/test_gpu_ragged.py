"""GPU parity of the search when the layers' configuration sets differ in size (Sec. 3: one set
per layer; Sec. 5: a set per layer type), against the oracle's Alg. 1 for such tables."""
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


def run_ragged(ctx, n_nodes, edges, Cn, seed, hi, schedules=(wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD), lo=0):
    from paper_1802_04924_amd import UNDO_RECOMPUTE, UNDO_STORED
    edges = np.asarray(edges, np.int32).reshape(-1, 2)
    tc, ts, tx = wl.ragged_tables(n_nodes, edges, Cn, seed, lo, hi)
    d_tc, d_ts, d_tx = dev(tc), dev(ts), dev(tx)
    for schedule in schedules:
        ref = oracle.search_ragged(n_nodes, edges, Cn, tc, ts, tx, schedule)
        # small searches run as one launch of one workgroup unless told otherwise: both paths are checked
        # and rounds with little work run on the wavefront-per-tile kernel unless told otherwise: both kernels
        for single in ((True, False) if int(np.max(Cn)) <= 64 else (True,)):
            ctx.set_single_launch(single)
            for wave in (True, False):
                ctx.set_small_product_kernel(wave)
                for undo in (UNDO_STORED, UNDO_RECOMPUTE):
                    cost, S = ctx.search_graph_ragged(n_nodes, edges, Cn, d_tc, d_ts, d_tx, schedule, undo)
                    assert cost == ref["cost"], (schedule, undo, single, wave)
                    assert np.array_equal(S, ref["strategy"]), (schedule, undo, single, wave)
        ctx.set_single_launch(True)
        ctx.set_small_product_kernel(True)
        assert oracle.strategy_cost_ragged(n_nodes, edges, Cn, tc, ts, tx, S) == cost
        assert (S >= 0).all() and (S < np.asarray(Cn)).all()
    return cost, S


@pytest.mark.parametrize("n_layers,c_min,c_max,hi", [
    (2, 1, 9, 50), (3, 100, 300, 1000), (12, 1, 40, 3), (25, 60, 200, 1 << 20), (7, 120, 270, 1 << 24),
    (40, 1, 3, 7),
])
def test_ragged_chains(ctx, n_layers, c_min, c_max, hi):
    # (searches below 2^29 cell updates: no read-back of value ranges, plain and value-only variants)
    Cn = wl.ragged_counts(n_layers, n_layers + c_max, c_min, c_max)
    run_ragged(ctx, n_layers, wl.chain_edges(n_layers), Cn, seed=n_layers, hi=hi)


def test_ragged_round_with_thousands_of_small_tiles(ctx):
    # first round: 29 products of about 130^3 -- little enough work for the wavefront-per-tile kernel,
    # enough output (over 2048 tiles of 16 x 16) for its larger tile; shapes differ from product to product
    Cn = wl.ragged_counts(60, 61, 100, 160)
    run_ragged(ctx, 60, wl.chain_edges(60), Cn, seed=60, hi=1 << 18, schedules=(wl.SCHEDULE_ROUNDS,))


def test_ragged_rounds_of_a_few_products_with_long_rows(ctx):
    # rounds of 4, 2, 1 products of about 200^3, every shape its own: a few hundred tiles of 16 x 16 and
    # rows of 201 to 290 candidates, where four wavefronts share a 16 x 16 tile, each with a ragged
    # quarter of the candidates; heavy ties (hi = 2) and none
    Cn = np.array([211, 270, 250, 283, 222, 295, 201, 249, 204], np.int32)
    for hi in (2, 1 << 20):
        run_ragged(ctx, 9, wl.chain_edges(9), Cn, seed=9 + hi, hi=hi)


@pytest.mark.parametrize("big,hi", [(600, 1 << 16), (900, 1 << 16), (900, 1 << 28)])
def test_ragged_small_round_feeds_a_large_one(ctx, big, hi):
    # first round of the search: two products of big x 4 x big (the wavefront-per-tile kernel); second: one
    # product of big^3 on the tiled kernel (compare/select at 600, packed keys at 900: 2^29 cell updates and
    # more), whose operands are both outputs of the first -- their value ranges must have been measured there
    Cn = np.array([big, 4, big, 4, big], np.int32)
    run_ragged(ctx, 5, wl.chain_edges(5), Cn, seed=big, hi=hi, schedules=(wl.SCHEDULE_ROUNDS,))


def test_ragged_against_exhaustive_definition(ctx):
    from oracle import brute
    edges = np.array([(0, 1), (1, 2), (0, 2), (2, 3), (3, 4), (2, 4)], np.int32)
    Cn = np.array([3, 7, 2, 5, 4], np.int32)
    tc, ts, tx = wl.ragged_tables(5, edges, Cn, 5, 0, 30)
    cost, S = ctx.search_graph_ragged(5, edges, Cn, dev(tc), dev(ts), dev(tx))
    best, _, _ = brute.brute_force_ragged(5, edges, Cn, tc, ts, tx)
    assert cost == best
    assert oracle.strategy_cost_ragged(5, edges, Cn, tc, ts, tx, S) == best


def test_ragged_by_layer_type(ctx):
    # a VGG-shaped chain: convolutions with many configurations, pooling with fewer, the
    # fully-connected tail with few (Sec. 5: the configuration set depends on the layer type)
    kinds = "ccpccpcccpcccpcccpfff"
    Cn = np.array([{"c": 163, "p": 40, "f": 24}[k] for k in kinds], np.int32)
    run_ragged(ctx, len(kinds), wl.chain_edges(len(kinds)), Cn, seed=16, hi=100000)


@pytest.mark.parametrize("modules,c_min,c_max,hi", [(1, 1, 6, 3), (2, 20, 70, 100000), (6, 30, 140, 1 << 18)])
def test_ragged_forkjoin(ctx, modules, c_min, c_max, hi):
    n, edges = wl.forkjoin_edges(modules, modules)
    Cn = wl.ragged_counts(n, 3 * modules + c_max, c_min, c_max)
    run_ragged(ctx, n, edges, Cn, seed=modules, hi=hi)


@pytest.mark.parametrize("seed", range(6))
def test_ragged_random_series_parallel(ctx, seed):
    from paper_1802_04924_amd import plan_graph
    n, edges = wl.series_parallel_edges(25 + 6 * seed, seed, p_branch=0.08 if seed % 2 else 0.0)
    c_max = [4, 30, 90][seed % 3]
    Cn = wl.ragged_counts(n, 100 + seed, 1, c_max)
    if plan_graph(n, edges)["n_residual_nodes"] > 2 and float(c_max) ** plan_graph(n, edges)["n_residual_nodes"] > (1 << 32):
        Cn = wl.ragged_counts(n, 100 + seed, 1, 3)          # possibly more strategies than either side enumerates
    run_ragged(ctx, n, edges, Cn, seed=seed, hi=[2, 1000, 1 << 20][seed % 3])


IRREDUCIBLE = {
    "star_out": (4, [(0, 1), (0, 2), (0, 3)]),
    "star_in": (4, [(1, 0), (2, 0), (3, 0)]),
    "bipartite": (4, [(0, 2), (0, 3), (1, 2), (1, 3)]),
    "two_towers": (7, [(0, 1), (1, 4), (2, 3), (3, 4), (4, 5), (5, 6), (4, 6)]),
    "mixed_components": (8, [(0, 1), (0, 2), (0, 3), (4, 5), (5, 6), (7, 6)]),
}


@pytest.mark.parametrize("name", sorted(IRREDUCIBLE))
@pytest.mark.parametrize("c_max,hi", [(2, 1), (9, 3), (40, 1000)])
def test_ragged_residual_components_use_mixed_radix(ctx, name, c_max, hi):
    n, e = IRREDUCIBLE[name]
    Cn = wl.ragged_counts(n, c_max + len(e), 1, c_max)
    run_ragged(ctx, n, e, Cn, seed=c_max, hi=hi)


def test_ragged_small_irregular_graphs(ctx):
    graphs = {
        "single": (1, []), "two_isolated": (2, []), "parallel3": (2, [(0, 1), (0, 1), (0, 1)]),
        "diamond_skip": (4, [(0, 1), (0, 2), (1, 3), (2, 3), (0, 3)]),
        "backward_ids": (4, [(3, 1), (1, 0), (0, 2)]),
        "two_chains": (6, [(0, 1), (1, 2), (3, 4), (4, 5)]),
    }
    for name, (n, e) in graphs.items():
        for c_max, hi in ((1, 9), (5, 2), (70, 1000)):
            Cn = wl.ragged_counts(n, n + c_max, 1, c_max)
            run_ragged(ctx, n, e, Cn, seed=3, hi=hi)


def test_ragged_negative_costs_and_wide_ranges(ctx):
    # values of both signs; ranges wide enough that the packed-key variant does not apply
    Cn = wl.ragged_counts(9, 9, 50, 150)
    run_ragged(ctx, 9, wl.chain_edges(9), Cn, seed=4, hi=1 << 26, lo=-(1 << 26))


def test_constant_counts_equal_the_uniform_call(ctx):
    from paper_1802_04924_amd import search_workspace_bytes, search_workspace_bytes_ragged
    p = wl.forkjoin_problem(2, 48, seed=9, lo=0, hi=5000)
    Cn = np.full(p["n_nodes"], 48, np.int32)
    d = dev(p["tc"]), dev(p["ts"]), dev(p["tx"])
    a = ctx.search_graph(p["n_nodes"], p["edges"], 48, *d)
    b = ctx.search_graph_ragged(p["n_nodes"], p["edges"], Cn, d[0].reshape(-1), d[1].reshape(-1), d[2].reshape(-1))
    assert a[0] == b[0] and np.array_equal(a[1], b[1])
    for undo in (0, 1):
        assert search_workspace_bytes(p["n_nodes"], p["edges"], 48, 0, undo) == \
            search_workspace_bytes_ragged(p["n_nodes"], p["edges"], Cn, 0, undo) > 0


def test_ragged_invalid_counts_are_refused(ctx):
    import ctypes
    from paper_1802_04924_amd import binding, search_workspace_bytes_ragged
    lib, h = binding.load(), ctx._h
    t = dev(np.zeros(64, np.int32))
    p = ctypes.c_void_p(t.data_ptr())
    e = np.array([[0, 1]], np.int32)
    cost = ctypes.c_int32(7)
    S = np.full(2, -5, np.int32)
    for bad in ([0, 3], [3, -1], [3, 65537]):
        Cn = np.array(bad, np.int32)
        rc = lib.lwp_search_graph_ragged(h, 2, 1, e.ctypes.data, Cn.ctypes.data, p, p, p, 0, 0, ctypes.byref(cost), S.ctypes.data)
        assert rc == binding.E_INVAL
        assert search_workspace_bytes_ragged(2, e, Cn) == 0
    assert lib.lwp_search_graph_ragged(h, 2, 1, e.ctypes.data, None, p, p, p, 0, 0, ctypes.byref(cost), S.ctypes.data) == binding.E_INVAL
    assert cost.value == 7 and (S == -5).all()
    # a residual component whose strategies exceed 2^32 is refused, a smaller one is not
    star = np.array([(0, 1), (0, 2), (0, 3)], np.int32)
    assert search_workspace_bytes_ragged(4, star, [65536, 65536, 2, 1]) == 0
    assert search_workspace_bytes_ragged(4, star, [65536, 65536, 1, 1]) > 0


# ---- cost tables from per-layer configuration lists (Sec. 4 / Table 1, Sec. 5.1) ----------------
def layer_lists(layers, n_devices):
    from paper_1802_04924_amd import enumerate_configs
    lists = [enumerate_configs(l, n_devices) for l in layers]
    return np.concatenate(lists), np.array([len(x) for x in lists], np.int32)


@pytest.mark.parametrize("net", ["alexnet", "vgg16"])
def test_ragged_cost_tables_and_search(ctx, net):
    layers = wl.alexnet_layers(256) if net == "alexnet" else wl.vgg16_layers(64)
    edges = wl.chain_edges(len(layers))
    m = wl.machine()
    configs, Cn = layer_lists(layers, m["n_devices"])
    assert Cn.max() == 163 and Cn.min() == 57
    tc, ts, tx = ctx.build_cost_tables_ragged(layers, edges, configs, Cn, m)
    rtc, rts, rtx = oracle.build_cost_tables_ragged(layers, edges, configs, Cn, m)
    assert np.array_equal(tc.cpu().numpy(), rtc)
    assert np.array_equal(ts.cpu().numpy(), rts)
    assert np.array_equal(tx.cpu().numpy(), rtx)
    for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
        ref = oracle.search_ragged(len(layers), edges, Cn, rtc, rts, rtx, schedule)
        for undo in (0, 1):
            cost, S = ctx.search_graph_ragged(len(layers), edges, Cn, tc, ts, tx, schedule, undo)
            assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])
    # the same optimum as with one padded list of 256 rows for all layers
    full = wl.config_table(16, 256)
    utc, uts, utx = ctx.build_cost_tables(layers, edges, full, m)
    ucost, uS = ctx.search_graph(len(layers), edges, 256, utc, uts, utx)
    off = np.concatenate([[0], np.cumsum(Cn)])
    assert ucost == cost
    for l in range(len(layers)):
        assert tuple(full[uS[l]][:5]) == tuple(configs[off[l] + S[l]][:5])


def test_ragged_cost_tables_odd_shapes(ctx):
    N = 6
    layers = np.asarray([
        (wl.KIND_CONV, N, 3, 23, 31, 10, 12, 16, 3, 3, 2, 2, 1, 1),
        (wl.KIND_POOL, N, 10, 12, 16, 10, 6, 8, 2, 2, 2, 2, 0, 0),
        (wl.KIND_CONV, N, 10, 6, 8, 7, 6, 8, 5, 3, 1, 1, 2, 1),
        (wl.KIND_POOL, N, 7, 6, 8, 7, 4, 6, 3, 3, 1, 1, 0, 0),
        (wl.KIND_FC, N, 7, 4, 6, 9, 1, 1, 4, 6, 1, 1, 0, 0),
        (wl.KIND_FC, N, 9, 1, 1, 5, 1, 1, 1, 1, 1, 1, 0, 0),
        (wl.KIND_CONV, N, 10, 6, 8, 7, 6, 8, 1, 1, 1, 1, 0, 0),
    ], np.int32)
    edges = np.array([[0, 1], [1, 2], [2, 3], [3, 4], [4, 5], [1, 6], [6, 3]], np.int32)
    m = {"n_devices": 12, "flop_per_ns": 7, "byte_per_ns": 3, "invalid_cost": 1 << 27}
    configs, Cn = layer_lists(layers, 12)
    # lists need not come from the enumeration: append rows the layer cannot use and non-power-of-two degrees
    extra = np.asarray([(3, 1, 1, 1, 0, 0), (1, 3, 2, 1, 6, 0), (0, 0, 0, 0, 0, 0), (16, 1, 1, 1, 0, 0)], np.int32)
    off = np.concatenate([[0], np.cumsum(Cn)])
    configs = np.concatenate([np.concatenate([configs[off[l]:off[l + 1]], extra[:1 + l % 4]]) for l in range(len(layers))])
    Cn = Cn + 1 + np.arange(len(layers), dtype=np.int32) % 4
    tc, ts, tx = ctx.build_cost_tables_ragged(layers, edges, configs, Cn, m)
    rtc, rts, rtx = oracle.build_cost_tables_ragged(layers, edges, configs, Cn, m)
    assert np.array_equal(tc.cpu().numpy(), rtc)
    assert np.array_equal(ts.cpu().numpy(), rts)
    assert np.array_equal(tx.cpu().numpy(), rtx)
    ref = oracle.search_ragged(len(layers), edges, Cn, rtc, rts, rtx)
    cost, S = ctx.search_graph_ragged(len(layers), edges, Cn, tc, ts, tx)
    assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])


def test_ragged_cost_tables_errors(ctx):
    from paper_1802_04924_amd import LwpError, binding
    layers = wl.alexnet_layers(8)
    edges = wl.chain_edges(len(layers))
    configs, Cn = layer_lists(layers, 4)
    m = wl.machine(n_devices=4)
    with pytest.raises(ValueError):
        ctx.build_cost_tables_ragged(layers, edges, configs, Cn[:-1], m)
    bad = layers.copy()
    bad[3, 2] += 1                                    # input channels no longer match the producer
    with pytest.raises(LwpError) as e:
        ctx.build_cost_tables_ragged(bad, edges, configs, Cn, m)
    assert e.value.code == binding.E_INVAL


@pytest.mark.parametrize("c_max,hi", [(5, 3), (120, 100000)])
def test_ragged_resnet_shaped(ctx, c_max, hi):
    n, edges = wl.resnet_edges(bottleneck=True)
    run_ragged(ctx, n, edges, wl.ragged_counts(n, c_max, 1, c_max), seed=c_max, hi=hi)


@pytest.mark.parametrize("hi,t_c_scale", [(1000, 1), (1 << 20, 1), (1 << 20, 400)])
def test_ragged_searches_large_enough_for_packed_keys(ctx, hi, t_c_scale):
    # launches of mixed shapes pick packed keys on the device (global offsets, or re-based per row when
    # node costs range widely); the last rounds, one product each, are small enough for the
    # wavefront-per-tile kernel (compare/select)
    Cn = wl.ragged_counts(10, 77, 350, 620)
    edges = wl.chain_edges(10)
    tc, ts, tx = wl.ragged_tables(10, edges, Cn, hi % 97, 0, hi)
    tc = (tc.astype(np.int64) * t_c_scale).astype(np.int32)
    from paper_1802_04924_amd import UNDO_STORED
    for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
        ref = oracle.search_ragged(10, edges, Cn, tc, ts, tx, schedule)
        ctx.profile_enable(True)
        ctx.profile_reset()
        cost, S = ctx.search_graph_ragged(10, edges, Cn, dev(tc), dev(ts), dev(tx), schedule, UNDO_STORED)
        prof = ctx.profile_read()
        ctx.profile_enable(False)
        assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])
        assert prof["products_keyed"] + prof["products_keyed_row"] + prof["products_plain"] == 8
        if schedule == wl.SCHEDULE_ROUNDS:       # the first round: four products in one launch of mixed shapes
            assert prof["products_keyed"] + prof["products_keyed_row"] >= 4
    n, fj = wl.forkjoin_edges(2, 3)
    Cn = wl.ragged_counts(n, 78, 250, 400)
    run_ragged(ctx, n, fj, Cn, seed=3, hi=hi, schedules=(wl.SCHEDULE_ROUNDS,))
