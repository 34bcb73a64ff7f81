"""A search prepared once (schedule, buffers, descriptors) and run many times must return, on
every run, what the one-shot search and the oracle return for the tables' contents at that moment."""
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


def replay_case(ctx, n, edges, Cn, schedule, seeds, hi):
    """One plan, several table contents written in place, other work of the context between the runs."""
    import torch
    edges = np.asarray(edges, np.int32).reshape(-1, 2)
    tc, ts, tx = wl.ragged_tables(n, edges, Cn, seeds[0], 0, hi)
    d_tc, d_ts, d_tx = dev(tc), dev(ts), dev(tx)
    other = wl.chain_problem(5, 40, 3)
    o_t = [dev(other[k]) for k in ("tc", "ts", "tx")]
    with ctx.search_plan(n, edges, Cn, d_tc, d_ts, d_tx, schedule) as plan:
        for rep, seed in enumerate(seeds):
            tc, ts, tx = wl.ragged_tables(n, edges, Cn, seed, 0, hi)
            d_tc.copy_(torch.from_numpy(tc)); d_ts.copy_(torch.from_numpy(ts))
            if len(tx):
                d_tx.copy_(torch.from_numpy(tx))
            ref = oracle.search_ragged(n, edges, Cn, tc, ts, tx, schedule)
            for again in range(2):                     # the same contents twice, then new contents
                cost, S = plan.run()
                assert cost == ref["cost"], (rep, again)
                assert np.array_equal(S, ref["strategy"]), (rep, again)
                # other searches of the same context and a synchronisation between runs
                ecost, eS = ctx.search_graph_ragged(n, edges, Cn, d_tc, d_ts, d_tx, schedule, 1)
                assert ecost == cost and np.array_equal(eS, S)
                ctx.search_graph(other["n_nodes"], other["edges"], other["C"], *o_t)
                torch.cuda.synchronize()


def test_plan_replays_chain(ctx):
    Cn = wl.ragged_counts(12, 5, 40, 200)
    for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
        replay_case(ctx, 12, wl.chain_edges(12), Cn, schedule, seeds=(1, 2, 3), hi=100000)


def test_plan_replays_forkjoin_with_edge_eliminations(ctx):
    n, edges = wl.forkjoin_edges(3, 1)
    replay_case(ctx, n, edges, np.full(n, 64, np.int32), wl.SCHEDULE_ROUNDS, seeds=(4, 5, 6, 7), hi=1 << 20)
    replay_case(ctx, n, edges, wl.ragged_counts(n, 9, 1, 90), wl.SCHEDULE_ROUNDS, seeds=(8, 9), hi=3)


def test_plan_replays_residual_enumeration(ctx):
    star = [(0, 1), (0, 2), (0, 3), (4, 5), (5, 6), (7, 6)]
    replay_case(ctx, 8, star, wl.ragged_counts(8, 2, 1, 30), wl.SCHEDULE_ROUNDS, seeds=(1, 2, 3), hi=1000)
    replay_case(ctx, 1, [], np.array([17], np.int32), wl.SCHEDULE_ROUNDS, seeds=(1, 2), hi=9)


def test_plan_with_split_and_wide_ranges(ctx):
    # products large enough to split tiles over workgroups; values far beyond what packed keys hold
    Cn = np.array([300, 512, 257, 300], np.int32)
    replay_case(ctx, 4, wl.chain_edges(4), Cn, wl.SCHEDULE_ROUNDS, seeds=(11, 12, 13), hi=1 << 26)


def test_plan_reports_overflow_from_the_present_contents(ctx):
    import torch
    from paper_1802_04924_amd import LwpError, binding
    p = wl.chain_problem(6, 33, 5)
    d = [dev(p[k]) for k in ("tc", "ts", "tx")]
    with ctx.search_plan(6, p["edges"], 33, *d) as plan:
        cost, S = plan.run()
        ref = oracle.search(6, p["edges"], 33, p["tc"], p["ts"], p["tx"])
        assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])
        d[2].fill_((1 << 30) - 1)                      # sums of three such entries leave int32
        with pytest.raises(LwpError) as e:
            plan.run()
        assert e.value.code == binding.E_OVERFLOW
        d[2].copy_(torch.from_numpy(p["tx"]))          # and the plan is still usable afterwards
        cost2, S2 = plan.run()
        assert cost2 == cost and np.array_equal(S2, S)


def test_plan_uniform_count_and_errors(ctx):
    from paper_1802_04924_amd import LwpError, binding
    p = wl.forkjoin_problem(2, 48, seed=9, lo=0, hi=5000)
    d = [dev(p[k]) for k in ("tc", "ts", "tx")]
    with ctx.search_plan(p["n_nodes"], p["edges"], 48, *d) as plan:
        a = plan.run()
    b = ctx.search_graph(p["n_nodes"], p["edges"], 48, *d)
    assert a[0] == b[0] and np.array_equal(a[1], b[1])
    with pytest.raises(LwpError) as e:
        ctx.search_plan(3, [(0, 1), (1, 2), (2, 0)], 4, dev(np.zeros(12, np.int32)), dev(np.zeros(12, np.int32)),
                        dev(np.zeros(48, np.int32)))
    assert e.value.code == binding.E_GRAPH
