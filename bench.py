#!/usr/bin/env python3
"""Benchmark of the strategy search on one MI355X.

A step is one whole search (Alg. 1: all eliminations, residual solve, undo) over tables that
are already resident in HBM.  Default workload: the 64-layer chain with 4096 configurations per
layer (62 sequential 4096^3 node eliminations).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4|cfg3|cfg2|cfg0]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# VALU int32 peak of MI355X: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second.
# One cell update of Eq. 2 is one add and one min, i.e. 2 lane-operations.
PEAK_INT32_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
OPS_PER_UPDATE = 2
# L2<->fabric bytes of one 4096^3 min-plus launch from the rocprofv3 --pmc passes (FETCH_SIZE and
# WRITE_SIZE, each scaled by a 1 GiB reference copy): profiles/minplus_kernel_C4096_pmc.txt.
PMC_TRAFFIC_BYTES_C4096 = 1_775_358_427


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(kind, payload):
    """Times the CPU oracle, as it stands, on a bounded sample of the same workload."""
    import oracle
    threads = oracle.omp_threads()
    if kind == "search":
        p = payload
        t0 = time.perf_counter()
        oracle.search(p["n_nodes"], p["edges"], p["C"], p["tc"], p["ts"], p["tx"], p["schedule"])
        dt = time.perf_counter() - t0
        return {"value": p["updates"] / dt / 1e9, "unit": "G cell-updates/s", "cores": threads, "kind": "oracle",
                "sample": f"the whole search once ({dt * 1e3:.1f} ms)", "search_ms": dt * 1e3}
    if kind == "search_ragged":
        p = payload
        t0 = time.perf_counter()
        oracle.search_ragged(p["n_nodes"], p["edges"], p["Cn"], p["tc"], p["ts"], p["tx"], p["schedule"])
        dt = time.perf_counter() - t0
        return {"value": p["updates"] / dt / 1e9, "unit": "G cell-updates/s", "cores": threads, "kind": "oracle",
                "sample": f"the whole search once ({dt * 1e3:.1f} ms)", "search_ms": dt * 1e3}
    if kind == "fold":
        # the first eliminations of the left fold T <- T (x) B_j: as many as it takes to pass 10 s
        p = payload
        C = p["C"]
        w = (p["tc"] + p["ts"]).astype(np.int32)
        T = p["tx"][0]
        k = 0
        t0 = time.perf_counter()
        while k < p["n_nodes"] - 2 and time.perf_counter() - t0 < 10.0:
            k += 1
            T, _ = oracle.minplus_argmin(T, w[k], p["tx"][k])
        dt = time.perf_counter() - t0
        return {"value": k * C ** 3 / dt / 1e9, "unit": "G cell-updates/s", "cores": threads, "kind": "oracle",
                "sample": f"the first {k} of {p['n_nodes'] - 2} node eliminations of the left fold ({k * C ** 3:.3g} cell updates, {dt:.1f} s)"}
    A, w, B, what = payload
    # calibrate on a few rows, then size the sample to roughly 12 s
    probe = min(64, A.shape[0])
    t0 = time.perf_counter()
    oracle.minplus_argmin(A[:probe], w, B)
    rate = probe * B.shape[0] * B.shape[1] / (time.perf_counter() - t0)
    rows = int(max(probe, min(A.shape[0], 12.0 * rate / (B.shape[0] * B.shape[1]))))
    t0 = time.perf_counter()
    oracle.minplus_argmin(A[:rows], w, B)
    dt = time.perf_counter() - t0
    upd = rows * B.shape[0] * B.shape[1]
    return {"value": upd / dt / 1e9, "unit": "G cell-updates/s", "cores": threads, "kind": "oracle",
            "sample": f"{what}: first {rows} of {A.shape[0]} output rows ({upd:.3g} cell updates, {dt:.1f} s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg4", choices=["cfg0", "cfg1", "cfg2", "cfg3", "cfg4", "resid", "vgg16", "cfg1-lists", "vgg16-lists", "wide"],
                    help="cfg4 is the headline; *-lists: the AlexNet- / VGG-16-shaped chain with one configuration "
                         "list per layer (Sec. 4, Table 1) instead of one padded list of 256 rows; wide: a chain "
                         "with node costs from microseconds to half a second (no global offset fits packed keys)")
    ap.add_argument("--layers", type=int, default=64, help="cfg4 only: chain length")
    ap.add_argument("--configs", type=int, default=0, help="override C of the workload")
    ap.add_argument("--undo", default="stored", choices=["stored", "recompute"],
                    help="undo pass: look up stored argmin tables, or recompute the argmin as Alg. 1 does")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-events", action="store_true",
                    help="diagnostic: do not bracket the elimination launches with HIP events (no roofline figures)")
    ap.add_argument("--replay", action="store_true",
                    help="prepare the search once (schedule, buffers, descriptors; recomputed undo) and time runs of "
                         "the prepared plan")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch
    from paper_1802_04924_amd import Context, workloads as wl
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    torch.cuda.set_device(0)

    def dev(a):
        return torch.from_numpy(a).cuda()

    t_gen = time.perf_counter()
    name = args.workload
    if name == "cfg3":
        C = args.configs or 256
        batch = 4096
        A, w, B = wl.config3(batch, C)
        dA, dw, dB = dev(A), dev(w), dev(B)
        out = torch.empty((batch, C, C), dtype=torch.int32, device="cuda")
        arg = torch.empty_like(out)
        updates = batch * C ** 3
        workload = f"cfg3: {batch} independent {C}^3 min-plus+argmin products, values in [0,2^20], seed 3"
        ctx = Context(0)

        def step():
            ctx.eliminate_node(dA, dw, dB, out=out, argmin=arg)
            ctx.synchronize()
        # rows of many A tables against one (w, B): the same loop nest as whole products, sized to ~12 s
        cpu_payload = ("minplus", (A.reshape(batch * C, C), w[0], B[0], "rows of the A tables against (w[0], B[0])"))
    elif name.endswith("-lists"):
        from paper_1802_04924_amd import enumerate_configs, plan_graph
        p = wl.config1() if name == "cfg1-lists" else wl.vgg16_problem()
        lists = [enumerate_configs(l, p["machine"]["n_devices"]) for l in p["layers"]]
        Cn = np.array([len(x) for x in lists], np.int32)
        with Context(0) as c1:
            dtc, dts, dtx = c1.build_cost_tables_ragged(p["layers"], p["edges"], np.concatenate(lists), Cn, p["machine"])
        steps = plan_graph(p["n_nodes"], p["edges"], p["schedule"])["steps"]
        updates = int(sum(int(Cn[s["i"]]) * int(Cn[s["j"]]) * int(Cn[s["k"]]) for s in steps if s["kind"] == 0))
        workload = (f"{p['name'].rsplit('_', 1)[0]}_lists: {p['n_nodes']} nodes, {len(p['edges'])} edges, "
                    f"{int(Cn.min())}..{int(Cn.max())} configurations per layer, {p['n_nodes'] - 2} node eliminations")
        if args.undo == "recompute":
            workload += ", argmin recomputed in the undo pass"
        ctx = Context(0)
        result = {}

        def step():
            result["cost"], result["S"] = ctx.search_graph_ragged(p["n_nodes"], p["edges"], Cn, dtc, dts, dtx, p["schedule"],
                                                                  1 if args.undo == "recompute" else 0)
        plan_args = (p["n_nodes"], p["edges"], Cn, dtc.reshape(-1), dts.reshape(-1), dtx.reshape(-1), p["schedule"])
        q = {"n_nodes": p["n_nodes"], "edges": p["edges"], "Cn": Cn, "tc": dtc.cpu().numpy(), "ts": dts.cpu().numpy(),
             "tx": dtx.cpu().numpy(), "schedule": p["schedule"], "updates": updates}
        cpu_payload = ("search_ragged", q)
        C = int(Cn.max())
    else:
        if name == "cfg4":
            p = wl.config4(args.layers, args.configs or 4096)
        elif name in ("cfg1", "vgg16"):
            # tables of the AlexNet- / VGG-16-shaped chain come from the library's own cost-model kernels
            p = wl.config1() if name == "cfg1" else wl.vgg16_problem()
            with Context(0) as c1:
                tabs = c1.build_cost_tables(p["layers"], p["edges"], p["configs"], p["machine"])
            p["tc"], p["ts"], p["tx"] = (t.cpu().numpy() for t in tabs)
        elif name == "cfg2":
            p = wl.config2(args.configs or 512)
        elif name == "wide":
            Cw = args.configs or 2048
            p = wl.chain_problem(min(args.layers, 10), Cw, 6, tc_range=(1000, 1 << 29), ts_range=(0, 1 << 20),
                                 tx_range=(0, 1 << 22), schedule=wl.SCHEDULE_LEFT_FOLD, name=f"wide_chain_C{Cw}")
        elif name == "resid":
            # a graph no elimination applies to: one layer feeding three that never rejoin (K = 4);
            # the whole search is the enumeration of C^4 strategies of the final graph
            Cr = args.configs or 160
            e = np.array([[0, 1], [0, 2], [0, 3]], np.int32)
            tc, ts, tx = wl.random_tables(4, e, Cr, 7, (0, 1 << 20), (0, 1 << 20), (0, 1 << 20))
            p = {"name": f"resid_star4_C{Cr}", "n_nodes": 4, "edges": e, "C": Cr, "tc": tc, "ts": ts, "tx": tx,
                 "schedule": wl.SCHEDULE_ROUNDS}
        else:
            p = wl.config0()
        C = p["C"]
        dtc, dts, dtx = dev(p["tc"]), dev(p["ts"]), dev(p["tx"])
        n_elim = p["n_nodes"] - 2
        updates = n_elim * C ** 3
        workload = f"{p['name']}: {p['n_nodes']} nodes, {len(p['edges'])} edges, C={C}, {n_elim} node eliminations"
        if args.undo == "recompute":
            workload += ", argmin recomputed in the undo pass"
        if name == "resid":
            updates = C ** 4      # strategies enumerated, reported in the same field
            workload = f"{p['name']}: 4 residual nodes, C={C}, {updates:.3g} strategies enumerated per search"
        ctx = Context(0)
        result = {}

        def step():
            result["cost"], result["S"] = ctx.search_graph(p["n_nodes"], p["edges"], C, dtc, dts, dtx, p["schedule"],
                                                           1 if args.undo == "recompute" else 0)
        plan_args = (p["n_nodes"], p["edges"], C, dtc, dts, dtx, p["schedule"])
        if name == "cfg4":
            cpu_payload = ("fold", p)
        elif name == "resid":
            # the oracle enumerates at most 2^26 strategies: time it on the first 64 configurations
            q = dict(p, C=64, tc=np.ascontiguousarray(p["tc"][:, :64]), ts=np.ascontiguousarray(p["ts"][:, :64]),
                     tx=np.ascontiguousarray(p["tx"][:, :64, :64]), updates=64 ** 4)
            cpu_payload = ("search", q)
        else:
            p["updates"] = updates
            cpu_payload = ("search", p)
    if args.replay:
        if name == "cfg3":
            log("bench.py: --replay applies to the search workloads")
            sys.exit(2)
        plan = ctx.search_plan(*plan_args)
        workload += ", host-side work done once (argmin recomputed in the undo pass)"

        def step():  # noqa: F811
            result["cost"], result["S"] = plan.run()
    log(f"[bench] inputs ready in {time.perf_counter() - t_gen:.1f} s: {workload}")

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile_enable(not args.no_events)
    ctx.profile_reset()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    ms_per_step = dt / args.steps * 1e3
    value = updates / (dt / args.steps) / 1e9

    # the int32 VALU rate the device sustains on the kernel's own two instructions, register-only
    valu = ctx.measure_valu_rate()
    node_ms = prof["node_ms"] / max(prof["node_launches"], 1)
    upd_per_launch = prof["node_cell_updates"] / max(prof["node_launches"], 1)
    achieved = OPS_PER_UPDATE * upd_per_launch / (node_ms * 1e-3) / 1e12 if node_ms > 0 else 0.0
    roofline = {"bound": "alu", "kernel": "minplus_kernel", "achieved": achieved, "peak": PEAK_INT32_TOPS,
                "unit": "TOP/s (int32 add+min, 2 per cell update)", "frac": achieved / PEAK_INT32_TOPS,
                "traffic": PMC_TRAFFIC_BYTES_C4096 if (name == "cfg4" and C == 4096) else None,
                "launches": prof["node_launches"], "avg_launch_ms": node_ms,
                "cell_updates_per_launch": upd_per_launch, "keyed_launches": prof["keyed_launches"],
                "kernel_cell_updates_per_s_G": upd_per_launch / (node_ms * 1e-3) / 1e9 if node_ms > 0 else 0.0,
                "measured_valu_lane_TOPs": valu["lane_ops_per_s"] / 1e12,
                "measured_add_min3_cell_updates_per_s_G": valu["cell_updates_per_s"] / 1e9,
                "frac_of_measured_add_min3": (upd_per_launch / (node_ms * 1e-3)) / valu["cell_updates_per_s"] if node_ms > 0 else 0.0}

    line = {"metric": "min-plus cell-updates/s over the whole strategy search", "value": value, "unit": "G cell-updates/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
            "config": {"workload": workload, "search_latency_ms": ms_per_step},
            "roofline": roofline}
    if name != "cfg3":
        line["config"]["cost"] = int(result["cost"])
    if not args.no_cpu:
        log("[bench] timing the CPU oracle on a bounded sample ...")
        line["cpu_baseline"] = cpu_baseline(*cpu_payload)
    print(json.dumps(line), flush=True)
    if args.replay:
        plan.close()
    ctx.close()


if __name__ == "__main__":
    main()
