#!/usr/bin/env python3
"""Benchmark of the strategy search on one MI355X.

A step is one whole search (Alg. 1: all eliminations, residual solve, undo) over tables that
are already resident in HBM.  Headline workload: the 64-layer chain with 4096 configurations per
layer (62 sequential 4096^3 node eliminations).  Prints ONE JSON line; with the default workload
("all") the line also carries, under config.all, the latency, min-plus kernel rate and oracle parity
of the four smaller benchmark configurations.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|cfg4|cfg3|cfg2|cfg1|cfg0|...]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# VALU int32 peak of MI355X: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second.
PEAK_LANE_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# One cell update of Eq. 2 is one add and one min.  A three-way min retires two mins, so the fewest
# instructions a kernel can issue per update is 1 add + 1/2 min3 = 1.5: the issue ceiling is
# 39.32 / 1.5 = 26.2 T cell updates/s.  (Counting 2 operations per update against the same 39.32 T
# would let a kernel pass 1.0; that figure is kept as frac_2op.)
INSTR_PER_UPDATE = 1.5
PMC_SUMMARY = os.path.join(ROOT, "profiles", "minplus_kernel_C4096_pmc.txt")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def pmc_traffic_bytes():
    """HBM-side bytes of one 4096^3 min-plus launch as the committed rocprofv3 --pmc summary gives them."""
    try:
        m = re.search(r"^traffic_bytes_per_launch\s*=\s*(\d+)", open(PMC_SUMMARY).read(), re.M)
        return int(m.group(1)) if m else None
    except OSError:
        return None


def oracle_threads():
    import oracle
    return oracle.omp_threads()


def viterbi_chain(tc, ts, tx):
    """Layered shortest path: the optimum of Eq. 1 on a chain, by the textbook recurrence."""
    w = tc.astype(np.int64) + ts.astype(np.int64)
    d = w[0].copy()
    for l in range(1, len(w)):
        d = (d[:, None] + tx[l - 1]).min(axis=0) + w[l]
    return int(d.min())


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


class Workload:
    """One benchmark configuration with its tables resident on the device."""

    def __init__(self, name, args):
        import torch
        from paper_1802_04924_amd import Context, workloads as wl
        self.name, self.args = name, args
        self.ctx = Context(0)
        if args.tiled_only:
            self.ctx.set_small_product_kernel(False)
        self.result = {}
        self.plan = None
        undo = 1 if args.undo == "recompute" else 0

        def dev(a):
            return torch.from_numpy(np.ascontiguousarray(a)).cuda()

        if name == "cfg3":
            C = args.configs or 256
            batch = 4096
            A, w, B = wl.config3(batch, C)
            self.host = (A, w, B)
            dA, dw, dB = dev(A), dev(w), dev(B)
            out = torch.empty((batch, C, C), dtype=torch.int32, device="cuda")
            arg = torch.empty_like(out)
            self.out, self.arg = out, arg
            self.updates = batch * C ** 3
            self.workload = f"cfg3: {batch} independent {C}^3 min-plus+argmin products, values in [0,2^20], seed 3"
            # the benchmark states the range its tables are drawn from; the call that takes such a
            # promise (and checks it on the device) is the one timed, the call that measures the
            # ranges itself is reported beside it
            bounds = (0, 1 << 20, 0, 1 << 20, 0, 1 << 20)

            def step():
                self.ctx.eliminate_node(dA, dw, dB, out=out, argmin=arg, bounds=bounds)
                self.ctx.synchronize()

            def step_measured():
                self.ctx.eliminate_node(dA, dw, dB, out=out, argmin=arg)
                self.ctx.synchronize()
            self.step, self.step_measured = step, step_measured
            # rows of many A tables against one (w, B): the same loop nest as whole products, sized to ~12 s
            self.cpu_payload = ("minplus", (A.reshape(batch * C, C), w[0], B[0], "rows of the A tables against (w[0], B[0])"))
            self.C = C
            return
        if name.endswith("-lists"):
            from paper_1802_04924_amd import enumerate_configs, plan_graph
            p = wl.config1() if name == "cfg1-lists" else wl.vgg16_problem()
            p["machine"] = dict(p["machine"], n_devices=args.devices)
            lists = [enumerate_configs(l, p["machine"]["n_devices"]) for l in p["layers"]]
            Cn = np.array([len(x) for x in lists], np.int32)
            with Context(0) as c1:
                dtc, dts, dtx = c1.build_cost_tables_ragged(p["layers"], p["edges"], np.concatenate(lists), Cn, p["machine"])
            steps = plan_graph(p["n_nodes"], p["edges"], p["schedule"])["steps"]
            self.updates = int(sum(int(Cn[s["i"]]) * int(Cn[s["j"]]) * int(Cn[s["k"]]) for s in steps if s["kind"] == 0))
            self.workload = (f"{p['name'].rsplit('_', 1)[0]}_lists: {p['n_nodes']} nodes, {len(p['edges'])} edges, "
                             f"{args.devices} devices, {int(Cn.min())}..{int(Cn.max())} configurations per layer, "
                             f"{p['n_nodes'] - 2} node eliminations")

            def step():
                self.result["cost"], self.result["S"] = self.ctx.search_graph_ragged(p["n_nodes"], p["edges"], Cn, dtc, dts, dtx,
                                                                                     p["schedule"], undo)
            self.step = step
            self.plan_args = (p["n_nodes"], p["edges"], Cn, dtc.reshape(-1), dts.reshape(-1), dtx.reshape(-1), p["schedule"])
            q = {"n_nodes": p["n_nodes"], "edges": p["edges"], "Cn": Cn, "tc": dtc.cpu().numpy(), "ts": dts.cpu().numpy(),
                 "tx": dtx.cpu().numpy(), "schedule": p["schedule"], "updates": self.updates}
            self.cpu_payload = ("search_ragged", q)
            self.p = q
            self.C = int(Cn.max())
        else:
            if name == "cfg4":
                p = wl.config4(args.layers, args.configs or 4096)
            elif name in ("cfg1", "vgg16"):
                # tables of the AlexNet- / VGG-16-shaped chain come from the library's own cost-model kernels
                if args.configs:
                    raise SystemExit(f"bench.py: {name} takes its 256 configurations per layer from the cost model; --configs does not apply")
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
            elif name == "baseline":
                # the layer count Table 3 gives for LeNet-5; 40^6 strategies is what a 32-bit strategy index holds
                Cb = args.configs or 40
                p = wl.chain_problem(6, Cb, 6, tc_range=(0, 1 << 20), ts_range=(0, 1 << 20), tx_range=(0, 1 << 20),
                                     schedule=wl.SCHEDULE_NONE, name=f"baseline_chain6_C{Cb}")
            else:
                p = wl.config0()
            C = p["C"]
            dtc, dts, dtx = dev(p["tc"]), dev(p["ts"]), dev(p["tx"])
            n_elim = p["n_nodes"] - 2
            self.updates = n_elim * C ** 3
            self.workload = f"{p['name']}: {p['n_nodes']} nodes, {len(p['edges'])} edges, C={C}, {n_elim} node eliminations"
            if name == "baseline":
                self.updates = C ** 6      # strategies enumerated, reported in the same field
                self.workload = (f"{p['name']}: no eliminations, {self.updates:.3g} strategies of the original graph enumerated "
                                 "per search")
            if name == "resid":
                self.updates = C ** 4      # strategies enumerated, reported in the same field
                self.workload = f"{p['name']}: 4 residual nodes, C={C}, {self.updates:.3g} strategies enumerated per search"

            def step():
                self.result["cost"], self.result["S"] = self.ctx.search_graph(p["n_nodes"], p["edges"], C, dtc, dts, dtx,
                                                                              p["schedule"], undo)
            self.step = step
            self.plan_args = (p["n_nodes"], p["edges"], C, dtc, dts, dtx, p["schedule"])
            p["updates"] = self.updates
            self.cpu_payload = ("fold", p) if name == "cfg4" else ("search", p)
            self.p = p
            self.C = C
        if args.undo == "recompute":
            self.workload += ", argmin recomputed in the undo pass"
        if args.replay:
            self.plan = self.ctx.search_plan(*self.plan_args)
            self.workload += ", host-side work done once (argmin recomputed in the undo pass)"

            def step_replay():
                self.result["cost"], self.result["S"] = self.plan.run()
            self.step = step_replay

    def parity(self):
        """The device's result against the oracle (in full where that takes seconds)."""
        import oracle
        if self.name == "cfg3":
            A, w, B = self.host
            oracle_s = 0.0
            for fn, what in ((self.step, "promised ranges"), (self.step_measured, "measured ranges")):
                self.out.zero_(); self.arg.zero_()
                fn()
                out, arg = self.out.cpu().numpy(), self.arg.cpu().numpy()
                for b in range(A.shape[0]):
                    t0 = time.perf_counter()
                    ro, ra = oracle.minplus_argmin(A[b], w[b], B[b])
                    oracle_s += time.perf_counter() - t0
                    if not (np.array_equal(out[b], ro) and np.array_equal(arg[b], ra)):
                        return {"ok": False, "how": f"product {b} differs from the oracle ({what})"}
            return {"ok": True, "oracle_ms": oracle_s / 2 * 1e3,
                    "how": f"all {A.shape[0]} products, minima and argmins, equal to the oracle's on both entry points"}
        self.step()
        cost, S = self.result["cost"], self.result["S"]
        p = self.p
        if self.name == "cfg4":
            ok = cost == viterbi_chain(p["tc"], p["ts"], p["tx"]) and \
                oracle.strategy_cost(p["n_nodes"], p["edges"], p["C"], p["tc"], p["ts"], p["tx"], S) == cost
            return {"ok": bool(ok), "how": "cost equals the layered shortest path and Eq. 1 of the returned strategy "
                                           "(the oracle's whole search takes minutes; the test-suite checks every elimination)"}
        t0 = time.perf_counter()
        if "Cn" in p:
            ref = oracle.search_ragged(p["n_nodes"], p["edges"], p["Cn"], p["tc"], p["ts"], p["tx"], p["schedule"])
        elif self.name == "resid" and p["C"] ** 4 > (1 << 32):
            return {"ok": None, "how": "more strategies than the oracle enumerates"}
        else:
            ref = oracle.search(p["n_nodes"], p["edges"], p["C"], p["tc"], p["ts"], p["tx"], p["schedule"])
        oracle_ms = (time.perf_counter() - t0) * 1e3
        ok = cost == ref["cost"] and np.array_equal(S, ref["strategy"])
        return {"ok": bool(ok), "oracle_ms": oracle_ms, "how": "cost and every configuration equal to the oracle's whole search"}

    def close(self):
        if self.plan is not None:
            self.plan.close()
        self.ctx.close()


def timed(fn, steps, warmup):
    """Per-step seconds of `steps` runs after `warmup` untimed ones, bracketed by synchronisations."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    per = []
    t_all = time.perf_counter()
    for _ in range(steps):
        t0 = time.perf_counter()
        fn()
        per.append(time.perf_counter() - t0)
    torch.cuda.synchronize()
    return (time.perf_counter() - t_all) / steps, per


def kernel_rate(wk, fn, steps):
    """Min-plus launches of `steps` runs of fn bracketed by HIP events on the library's stream."""
    import torch
    wk.ctx.profile_enable(True)
    wk.ctx.profile_reset()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    prof = wk.ctx.profile_read()
    wk.ctx.profile_enable(False)
    return prof


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="all",
                    choices=["all", "cfg0", "cfg1", "cfg2", "cfg3", "cfg4", "resid", "baseline", "vgg16", "cfg1-lists", "vgg16-lists", "wide"],
                    help="all: cfg4 as the headline plus latency, kernel rate and parity of cfg0..cfg3; *-lists: the AlexNet- / "
                         "VGG-16-shaped chain with one configuration list per layer (Sec. 4, Table 1) instead of one padded list "
                         "of 256 rows; wide: a chain with node costs from microseconds to half a second (no global offset fits "
                         "packed keys); baseline: the exhaustive search the paper compares with (Sec. 5.2, Table 3) on a 6-layer chain "
                         "with 40 configurations, every one of the 4.1e9 strategies enumerated")
    ap.add_argument("--layers", type=int, default=64, help="cfg4 only: chain length")
    ap.add_argument("--devices", type=int, default=16,
                    help="*-lists only: devices of the machine the configurations are enumerated for (the paper's Table 3 "
                         "searches are for 4 GPUs)")
    ap.add_argument("--configs", type=int, default=0, help="override C of the workload")
    ap.add_argument("--undo", default="stored", choices=["stored", "recompute"],
                    help="undo pass: look up stored argmin tables, or recompute the argmin as Alg. 1 does")
    ap.add_argument("--tiled-only", action="store_true",
                    help="keep every node elimination on the tiled kernel (no wavefront-per-tile kernel for small rounds)")
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
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    torch.cuda.set_device(0)
    headline = "cfg4" if args.workload == "all" else args.workload
    if args.replay and headline == "cfg3":
        log("bench.py: --replay applies to the search workloads")
        sys.exit(2)

    # ---- the smaller configurations: latency, kernel rate, parity against the oracle in full ----
    others = {}
    if args.workload == "all":
        sub = argparse.Namespace(**{**vars(args), "configs": 0, "layers": 64, "replay": False})
        for name in ("cfg0", "cfg1", "cfg2", "cfg3"):
            t_gen = time.perf_counter()
            wk = Workload(name, sub)
            # (cfg3: a launch of 3 ms; after the seconds of input generation on the host the clocks need some
            # launches to come up, so ten warm-up calls go first)
            n = 20 if name == "cfg3" else 30
            _, per = timed(wk.step, n, 10 if name == "cfg3" else 3)
            prof = kernel_rate(wk, wk.step, 3)
            entry = {"workload": wk.workload, "search_ms": statistics.median(per) * 1e3,
                     "whole_G_cell_updates_per_s": wk.updates / statistics.median(per) / 1e9,
                     "minplus_launches_per_search": prof["node_launches"] // 3,
                     "kernel_T_cell_updates_per_s": (prof["node_cell_updates"] / (prof["node_ms"] * 1e-3) / 1e12) if prof["node_ms"] > 0 else None}
            if entry["kernel_T_cell_updates_per_s"]:
                entry["kernel_frac_of_issue_ceiling"] = entry["kernel_T_cell_updates_per_s"] * INSTR_PER_UPDATE / PEAK_LANE_TOPS
            if name == "cfg3":
                _, per_m = timed(wk.step_measured, n, 3)
                entry["search_ms_ranges_measured_on_device"] = statistics.median(per_m) * 1e3
            else:
                entry["cost"] = int(wk.result["cost"])
            par = wk.parity()
            entry["parity"] = par["ok"]
            entry["parity_how"] = par["how"]
            # the parity check runs the oracle on the whole configuration: its time on the host cores
            entry["oracle_ms"] = par.get("oracle_ms")
            entry["oracle_cores"] = oracle_threads()
            others[name] = entry
            wk.close()
            del wk
            torch.cuda.empty_cache()
            log(f"[bench] {name}: {entry['search_ms']:.3f} ms, parity {entry['parity']} ({time.perf_counter() - t_gen:.1f} s)")

    # ---- the headline workload ----
    t_gen = time.perf_counter()
    wk = Workload(headline, args)
    log(f"[bench] inputs ready in {time.perf_counter() - t_gen:.1f} s: {wk.workload}")
    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        wk.step()
    torch.cuda.synchronize()
    wk.ctx.profile_enable(not args.no_events)
    wk.ctx.profile_reset()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wk.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = wk.ctx.profile_read()
    wk.ctx.profile_enable(False)
    ms_per_step = dt / args.steps * 1e3
    value = wk.updates / (dt / args.steps) / 1e9

    # the int32 VALU rate the device sustains on the kernel's own two instructions, register-only
    valu = wk.ctx.measure_valu_rate()
    node_ms = prof["node_ms"] / max(prof["node_launches"], 1)
    upd_per_launch = prof["node_cell_updates"] / max(prof["node_launches"], 1)
    upd_per_s = upd_per_launch / (node_ms * 1e-3) if node_ms > 0 else 0.0
    achieved = INSTR_PER_UPDATE * upd_per_s / 1e12
    roofline = {"bound": "alu", "kernel": "minplus_kernel", "achieved": achieved, "peak": PEAK_LANE_TOPS,
                "unit": "T int32 lane-operations/s issued: 1 add + 1/2 three-way min = 1.5 per cell update "
                        "(peak = 256 CUs x 64 lanes x 2.4 GHz; issue ceiling 26.2 T cell updates/s)",
                "frac": achieved / PEAK_LANE_TOPS,
                "frac_2op": 2 * upd_per_s / 1e12 / PEAK_LANE_TOPS,
                "traffic": pmc_traffic_bytes() if (headline == "cfg4" and wk.C == 4096 and args.undo == "stored") else None,
                "algorithmic_bytes": (4 * (2 * wk.C * wk.C + wk.C) + 8 * wk.C * wk.C) if headline == "cfg4" else None,
                "launches": prof["node_launches"], "avg_launch_ms": node_ms,
                "cell_updates_per_launch": upd_per_launch, "products_by_variant": {k: prof[k] for k in ("products_keyed", "products_keyed_row", "products_plain", "products_value")},
                "kernel_cell_updates_per_s_G": upd_per_s / 1e9,
                "measured_valu_lane_TOPs": valu["lane_ops_per_s"] / 1e12,
                "measured_add_min3_cell_updates_per_s_G": valu["cell_updates_per_s"] / 1e9,
                "frac_of_measured_add_min3": upd_per_s / valu["cell_updates_per_s"] if node_ms > 0 else 0.0}

    line = {"metric": "min-plus cell-updates/s over the whole strategy search", "value": value, "unit": "G cell-updates/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
            "config": {"workload": wk.workload, "search_latency_ms": ms_per_step},
            "roofline": roofline}
    if headline != "cfg3":
        line["config"]["cost"] = int(wk.result["cost"])
    if args.workload == "all":
        par = wk.parity()
        line["config"]["parity"] = par["ok"]
        line["config"]["parity_how"] = par["how"]
        line["config"]["all"] = others
    if not args.no_cpu:
        log("[bench] timing the CPU oracle on a bounded sample ...")
        line["cpu_baseline"] = cpu_baseline(*wk.cpu_payload)
    print(json.dumps(line), flush=True)
    wk.close()


if __name__ == "__main__":
    main()
