#!/usr/bin/env python3
"""Benchmark of the batched max-flow feasibility path on one MI355X.

One "step" is one pass of the hot path over one batch: `fc_maxflow_batch` on the 16 384 problems
(1024 sinks x 16 candidate throughputs) of the largest benchmark configuration (1024 compute +
128 switch nodes, random out-degree-8 fabric) -- launch ordering, preflow initialisation, discharge
steps, relabeling, termination, one flow value per problem -- on the auxiliary network of the paper's
Section 5.2.  The topology is uploaded once, outside the timed region (its cost is reported as
`graph_upload_ms`); the problem arrays are resident in HBM when the clock starts.  The same problems
through `fc_feasible` (candidate x sink grid + the verdict reduction of Theorem 1) are timed beside it,
and so are the four smaller configurations.

Prints ONE JSON line.  Every figure quoted in README.md can be re-derived from it:
  value, ms_per_step            whole-step wall time over the timed region
  roofline                      the dominant kernel against the vector-issue roof that binds it, with the
                                algorithmic-bytes rate (with and without the per-problem init term) and the
                                HBM traffic the hardware counters measured beside it
  configs                       configs 1-4: solves/s for both entry points, counters, kernel time
  graph_upload_ms, search       ingest + per-sink tables, and the optimality search on top of it
  cpu_baseline, parity_vs_oracle
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# vector-issue roof: 256 CUs x 4 SIMDs, one wave64 instruction per 4 cycles (16 lanes per SIMD), 2.4 GHz
VALU_PEAK_GINSTR = 256 * 4 * 2.4 / 4


def algorithmic_bytes(stats, n_problems, n_with_source, m_with_source):
    """Bytes the method itself must move for the work one launch did, in the plain 32-bit layout that keeps all
    state in memory: per arc scan a residual (4) and a height (4); per push two residuals and two excesses (16);
    per relabel a height (4); per global relabel all residuals read and all heights written; per problem the
    private state (2m residuals, n heights + excesses) written once -- the init term, returned separately."""
    n, m = n_with_source, m_with_source
    init = n_problems * (2 * m * 4 + n * 8)
    dynamic = (8 * stats["arc_scans"] + 16 * stats["pushes"] + 4 * stats["relabels"] +
               8 * stats["gr_arc_scans"] + stats["global_relabels"] * 4 * n)
    return dynamic + init, init


def load_counters():
    """Per-launch hardware counters of the solver kernel from the committed rocprofv3 summaries."""
    path = os.path.join(ROOT, "profiles", "counters.json")
    try:
        return json.load(open(path))
    except Exception:
        return {}


def roofline_block(stats, kernel_ms, n_problems, n_src, m_src, hw):
    """`hw`: {"valu_wave_instructions": .., "hbm_bytes": ..} per launch from profiles/counters.json, or {}."""
    total, init = algorithmic_bytes(stats, n_problems, n_src, m_src)
    sec = kernel_ms * 1e-3
    valu = hw.get("valu_wave_instructions")
    hbm = hw.get("hbm_bytes")
    achieved = None if valu is None else valu / sec / 1e9
    return {
        # what binds the kernel (counters in profiles/): instruction issue, not memory -- all per-problem state is in LDS
        "bound": "alu", "achieved": achieved, "peak": VALU_PEAK_GINSTR, "unit": "G wave-instructions/s (vector ALU)",
        "frac": None if achieved is None else achieved / VALU_PEAK_GINSTR,
        "traffic": hbm,
        "kernel": "fc_push_relabel_kernel", "kernel_ms": kernel_ms,
        "kernel_ms_is": "mean HIP-event time of the solver kernel over launches that write no counters (stats_time_only)",
        "valu_wave_instructions_per_launch": valu,
        "hbm": {
            "note": "algorithmic bytes = what a plain 32-bit in-memory layout would move for the counted work; the kernel "
                    "keeps that state in LDS, so measured HBM traffic is a small fraction of it",
            "algorithmic_bytes_per_launch": int(total), "algorithmic_init_bytes": int(init),
            "algorithmic_gbs": total / sec / 1e9, "algorithmic_frac_of_peak": total / sec / 1e9 / HBM_PEAK_GBS,
            "algorithmic_frac_without_init": (total - init) / sec / 1e9 / HBM_PEAK_GBS,
            "measured_bytes_per_launch": hbm,
            "measured_gbs": None if hbm is None else hbm / sec / 1e9,
            "measured_frac_of_peak": None if hbm is None else hbm / sec / 1e9 / HBM_PEAK_GBS,
            "peak_gbs": HBM_PEAK_GBS,
        },
    }


def _cpu_model():
    """Model name of the host CPU the oracle is timed on (first entry of /proc/cpuinfo), or 'unknown'."""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration 1..5 (default: the largest)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true",
                    help="headline and fc_feasible legs only (keeps profiler traces to the two kinds of launch)")
    ap.add_argument("--only", choices=["batch", "feasible"], default=None,
                    help="with --quick: time only this entry point (one kind of solver launch in a profile)")
    ap.add_argument("--back-end", type=str, default="3,4",
                    help="topologies for the switch-removal + tree-construction leg, comma-separated: config 3 and config 4 "
                         "(default, about 3 s together), 6 = the 1024-compute Eulerian switch fabric (about 20 s), 0 = skip")
    ap.add_argument("--threads-per-problem", type=int, default=0)
    ap.add_argument("--lanes-per-vertex", type=int, default=0)
    ap.add_argument("--copy-probe", action="store_true",
                    help="run a plain device copy of known size instead (calibrates the rocprofv3 HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (independent problems, no collectives); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as w
    from workloads.problems import config_candidates
    import paper_2402_06787_amd as fc

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if not os.path.exists(fc.LIB_PATH):
        from paper_2402_06787_amd import build as fcbuild
        fcbuild.build_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.copy_probe:
        nbytes = 1 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe": True, "bytes_read_per_copy": nbytes, "bytes_written_per_copy": nbytes,
                          "copies": 5}), flush=True)
        return

    hw_all = load_counters()
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)

    def timed(fn, warmup, steps):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def measure_config(cfg, steps, warmup, want=("batch", "feasible")):
        """Upload, search, and time both entry points on one configuration's problem list."""
        topo = w.config_topology(cfg)
        t0 = time.perf_counter()
        g = fc.fc_graph_upload(topo.n_vertices, topo.tail, topo.head, topo.bandwidth, topo.is_compute)
        upload_ms = (time.perf_counter() - t0) * 1e3
        t0 = time.perf_counter()                           # once more: without the first call's one-off costs (first large allocation, code objects)
        fc.fc_graph_upload(topo.n_vertices, topo.tail, topo.head, topo.bandwidth, topo.is_compute).close()
        upload_again_ms = (time.perf_counter() - t0) * 1e3
        info = fc.fc_graph_info(g)
        N = info.n_compute
        t0 = time.perf_counter()
        search = fc.fc_opt_throughput_search(g, 16)
        search_first_ms = (time.perf_counter() - t0) * 1e3     # may include loading code objects (first launches of the process)
        t0 = time.perf_counter()
        search = fc.fc_opt_throughput_search(g, 16)
        search_ms = (time.perf_counter() - t0) * 1e3
        inv = (search["inv_xstar"].numerator, search["inv_xstar"].denominator)
        cU, ck = config_candidates(cfg, inv)               # configs 2 and 5 centre their candidates on the optimum
        C = len(cU); P = C * N
        pl = w.all_sinks(topo, cU, ck)
        opts = {"src_cap_bound": int(ck.max())}
        if args.threads_per_problem:
            opts["threads_per_problem"] = args.threads_per_problem
        if args.lanes_per_vertex:
            opts["lanes_per_vertex"] = args.lanes_per_vertex
        n_src, m_src = topo.n_vertices + 1, info.n_arcs_merged + N
        d_sink, d_mult, d_cap = to_dev(pl.sink), to_dev(pl.edge_mult), to_dev(pl.src_cap)
        d_U, d_k = to_dev(cU), to_dev(ck)
        ws_b = torch.empty(max(256, fc.fc_maxflow_batch_workspace_bytes(g, P)), dtype=torch.uint8, device=dev)
        ws_f = torch.empty(max(256, fc.fc_feasible_workspace_bytes(g, C)), dtype=torch.uint8, device=dev)
        d_out = torch.empty(P, dtype=torch.int32, device=dev)
        batch = lambda **kw: fc.fc_maxflow_batch(g, d_sink, d_mult, d_cap, d_flow_out=d_out, d_workspace=ws_b,
                                                 options=dict(opts, **kw.pop("o", {})), **kw)
        feas = lambda **kw: fc.fc_feasible(g, d_U, d_k, want_witness=True, d_workspace=ws_f,
                                           options=dict(opts, **kw.pop("o", {})), **kw)
        res = {"config": cfg, "workload": f"{w.CONFIG_NAMES[cfg]}: {N} sinks x {C} candidates = {P} max-flows per step "
                                          f"(|V|={topo.n_vertices}, merged arcs={info.n_arcs_merged}, k={int(ck[0])}, "
                                          f"U={int(cU[0])}..{int(cU[-1])}, 1/x*={inv[0]}/{inv[1]})",
               "problems_per_step": P, "graph_upload_ms": upload_ms, "graph_upload_and_free_again_ms": upload_again_ms,
               "search": {"inv_xstar": f"{inv[0]}/{inv[1]}", "U": str(search["U"]), "k": search["k"], "rounds": search["rounds"],
                          "candidates_tested": search["trace_len"], "wall_ms": search_ms, "first_call_wall_ms": search_first_ms,
                          "incl_upload_ms": upload_ms + search_ms}}
        for name, fn in (("batch", batch), ("feasible", feas)):
            if name not in want:
                continue
            per_step = timed(lambda: fn(), warmup, steps)
            kms = []
            for _ in range(min(steps, 20)):                  # solver kernel alone, launches that write no counters
                r = fn(want_stats=True, o={"stats_time_only": 1})
                kms.append((r[1] if name == "batch" else r["stats"])["device_ms"])
            r = fn(want_stats=True)                          # one launch that counts its work
            st = r[1] if name == "batch" else r["stats"]
            for _ in range(3):
                fn()                                         # the cost hints as the plain path leaves them
            kernel_ms = float(np.mean(kms))
            entry = "fc_maxflow_batch" if name == "batch" else "fc_feasible"
            hw = hw_all.get(f"cfg{cfg}", {}).get(entry, {})
            res[entry] = {"value": P / per_step, "unit": "solves/s", "ms_per_step": per_step * 1e3,
                          "kernel_ms": kernel_ms, "kernel_ms_counting_launch": st["device_ms"],
                          "residual_edge_updates_per_sec": st["pushes"] / (kernel_ms * 1e-3),
                          "arc_scans_per_sec": st["arc_scans"] / (kernel_ms * 1e-3),
                          "per_launch": {k: int(v) for k, v in st.items() if k != "device_ms"},
                          "roofline": roofline_block(st, kernel_ms, P, n_src, m_src, hw)}
        handles = dict(g=g, topo=topo, info=info, N=N, P=P, C=C, cU=cU, ck=ck, pl=pl, opts=opts, d_U=d_U, d_k=d_k, ws_f=ws_f,
                       feas=feas, batch=batch, d_out=d_out, d_sink=d_sink, d_mult=d_mult, d_cap=d_cap, ws_b=ws_b)
        return res, handles

    # a first tiny upload + launch so that HIP initialisation and code-object loading are not billed to the ingest figure
    tw = w.config_topology(1)
    with fc.fc_graph_upload(tw.n_vertices, tw.tail, tw.head, tw.bandwidth, tw.is_compute) as g0:
        fc.fc_opt_throughput_search(g0, 4)
    torch.cuda.synchronize()

    cfg = args.config
    want = ("batch", "feasible") if not args.only else (args.only,)
    head, H = measure_config(cfg, args.steps, args.warmup, want)
    g, topo, N, P, C = H["g"], H["topo"], H["N"], H["P"], H["C"]
    cU, ck, opts, d_U, d_k, ws = H["cU"], H["ck"], H["opts"], H["d_U"], H["d_k"], H["ws_f"]
    main_leg = head["fc_maxflow_batch"] if "fc_maxflow_batch" in head else head["fc_feasible"]
    entry_point = "fc_maxflow_batch" if "fc_maxflow_batch" in head else "fc_feasible"

    out = {
        "metric": "max-flow solves/sec", "value": main_leg["value"], "unit": "solves/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_leg["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": head["workload"], "entry_point": entry_point, "problems_per_step": P},
        "residual_edge_updates_per_sec": main_leg["residual_edge_updates_per_sec"],
        "arc_scans_per_sec": main_leg["arc_scans_per_sec"],
        "kernel_ms": main_leg["kernel_ms"],
        "per_launch": main_leg["per_launch"],
        "roofline": main_leg["roofline"],
        "fc_feasible": head.get("fc_feasible") if entry_point != "fc_feasible" else None,
        "graph_upload_ms": head["graph_upload_ms"], "graph_upload_and_free_again_ms": head["graph_upload_and_free_again_ms"],
        "graph_upload_is": "fc_graph_upload: validation, merging, residual CSR on the host, copies, per-sink label / first-arc tables by a kernel on the device",
        "search": head["search"],
    }

    if not args.quick:
        # ---- the four smaller configurations, both entry points (a few ms each)
        out["configs"] = []
        for c in (1, 2, 3, 4):
            if c == cfg:
                continue
            r, h = measure_config(c, max(10, args.steps), max(3, args.warmup // 2))
            h["g"].close()
            out["configs"].append(r)

        # ---- the same step with the optional first-arc tree certificate (problems whose sink tree carries all
        # N*k units are answered without running the solver); reported beside the headline, never as it
        el = timed(lambda: H["feas"](o={"tree_certificate": 1}), args.warmup, args.steps)
        out["with_tree_certificate"] = {"value": P / el, "unit": "solves/s", "ms_per_step": el * 1e3,
                                        "note": "fc_feasible with option tree_certificate=1; not the headline"}
        for _ in range(3):                               # restore the cost hints the plain path leaves
            H["feas"]()
        torch.cuda.synchronize()

        # ---- in-place bandwidth updates (fc_graph_update_arcs) on a second copy of the graph: three links per call, as
        # one split of the edge-splitting loop changes, without and with the rebuild of the per-sink tables, and a
        # step of the same batch while the tables are off (every problem starts with a search for heights on the device)
        g2 = fc.fc_graph_upload(topo.n_vertices, topo.tail, topo.head, topo.bandwidth, topo.is_compute)
        ut, uh, ub = topo.tail[:3].copy(), topo.head[:3].copy(), topo.bandwidth[:3].copy()
        rp2, other2, pair2, bw2, fwd2 = fc.fc_graph_csr(g2)
        for i in range(3):                               # the merged bandwidth of each link; the calls set it one or two above that in turn
            rows = range(rp2[ut[i]], rp2[ut[i] + 1])
            ub[i] = next(int(bw2[r]) for r in rows if fwd2[r] and other2[r] == uh[i])
        def upd(refresh, bump):
            t0 = time.perf_counter()
            fc.fc_graph_update_arcs(g2, ut, uh, ub + bump, refresh_tables=refresh)
            return (time.perf_counter() - t0) * 1e3
        plain = [upd(False, 1 + (i & 1)) for i in range(20)]
        el_off = timed(lambda: fc.fc_maxflow_batch(g2, H["d_sink"], H["d_mult"], H["d_cap"], d_flow_out=H["d_out"], d_workspace=H["ws_b"],
                                                   options=opts), 3, 20)
        full = [upd(True, i & 1) for i in range(3)]
        g2.close()
        out["graph_update"] = {"links_per_call": 3, "ms_in_place": float(np.median(plain)), "ms_with_table_rebuild": float(np.median(full)),
                               "batch_without_tables": {"value": P / el_off, "unit": "solves/s", "ms_per_step": el_off * 1e3}}

        # ---- the fixed-k variant (Section 5.5, Algorithm 3) on the same topology: k = 2, 16 rational multipliers
        # around U*, capacities floor(U b_e)
        kfix = 2
        t0 = time.perf_counter()
        fk = fc.fc_fixed_k_search(g, kfix, 16)
        fk_ms = (time.perf_counter() - t0) * 1e3
        Us = fk["U_star"]
        f_num = np.array([max(1, Us.numerator - 8 + j) for j in range(16)], dtype=np.int32)
        f_den = np.full(16, Us.denominator, dtype=np.int32)
        f_k = np.full(16, kfix, dtype=np.int32)
        dn, dd, dk2 = (torch.from_numpy(a).to(dev) for a in (f_num, f_den, f_k))
        fopts = {"src_cap_bound": kfix}
        el = timed(lambda: fc.fc_feasible_floor(g, dn, dd, dk2, d_workspace=ws, options=fopts), args.warmup, args.steps)
        fixed = {"k": kfix, "U_star": f"{Us.numerator}/{Us.denominator}", "search_wall_ms": fk_ms,
                 "search_rounds": fk["rounds"], "value": 16 * N / el, "unit": "solves/s",
                 "ms_per_step": el * 1e3, "candidates": "16 multipliers (num - 8 + j) / den around U*"}
        if not args.no_cpu_baseline:
            import oracle
            fl = fc.fc_feasible_floor(g, dn, dd, dk2, want_flows=True, options=fopts)["flows"].cpu().numpy().astype(np.int64)
            pick = [0, 7, 8, 15]
            comp = np.flatnonzero(np.asarray(topo.is_compute)).astype(np.int32)
            ref = oracle.aux_maxflow_batch_floor(topo, np.tile(comp, len(pick)), np.repeat(f_num[pick], N),
                                                 np.repeat(f_den[pick], N), np.repeat(f_k[pick], N),
                                                 threads=max(1, min(16, os.cpu_count() or 1)))
            fixed["parity_vs_oracle"] = {"checked": int(ref.size), "mismatches": int((fl[pick].reshape(-1) != ref).sum())}
        out["fixed_k"] = fixed
        for _ in range(3):                               # restore the cost hints of the headline workload
            H["feas"]()
        torch.cuda.synchronize()

        # ---- edge-splitting gamma batches (Appendix E.2) on the DGX-A100-shaped config, which is Eulerian:
        # 256 (ingress, egress) pairs x 2N max-flows with explicit sources and unbounded arcs
        t3 = w.config_topology(3)
        g3 = fc.fc_graph_upload(t3.n_vertices, t3.tail, t3.head, t3.bandwidth, t3.is_compute)
        s3 = fc.fc_opt_throughput_search(g3, 16)
        U3, k3 = s3["U"].numerator, s3["k"] * s3["U"].denominator
        sw = np.flatnonzero(np.asarray(t3.is_compute) == 0)
        is_sw = np.zeros(t3.n_vertices, dtype=bool); is_sw[sw] = True
        tl, hd = np.asarray(t3.tail), np.asarray(t3.head)
        rng = np.random.default_rng(3)
        pu, pw, pt = [], [], []
        while len(pu) < 256:                             # random pairs e = (u, w), f = (w, t) through a switch w
            e = int(rng.integers(0, len(tl)))
            if not is_sw[hd[e]]:
                continue
            outs = np.flatnonzero(tl == hd[e])
            pu.append(int(tl[e])); pw.append(int(hd[e])); pt.append(int(hd[outs[int(rng.integers(0, len(outs)))]]))
        d3 = [to_dev(np.array(a, dtype=np.int32)) for a in (pu, pw, pt)]
        ws3 = torch.empty(fc.fc_split_gamma_workspace_bytes(g3, 256), dtype=torch.uint8, device=dev)
        reps = max(1, args.steps // 10)
        el = timed(lambda: fc.fc_split_gamma_batch(g3, U3, k3, *d3, d_workspace=ws3), 3, reps)
        P3 = 256 * 2 * t3.n_compute
        gamma = {"workload": f"{w.CONFIG_NAMES[3]} scaled by U={U3}, k={k3}: 256 pairs x 2N = {P3} max-flows per step",
                 "value": P3 / el, "unit": "solves/s", "ms_per_step": el * 1e3,
                 "note": "gamma only: a max-flow may stop once it cannot decide gamma any more, and is answered from the problem "
                         "without its compute node v where that one already got there (two launches)"}
        el = timed(lambda: fc.fc_split_gamma_batch(g3, U3, k3, *d3, want_flows=True, d_workspace=ws3), 3, reps)
        gamma["with_exact_flows"] = {"value": P3 / el, "unit": "solves/s", "ms_per_step": el * 1e3}
        if not args.no_cpu_baseline:
            import oracle
            got = fc.fc_split_gamma_batch(g3, U3, k3, *d3, d_workspace=ws3)["gamma"].cpu().numpy()
            D3 = w.Topology(t3.name, t3.n_vertices, t3.tail, t3.head,
                            (np.asarray(t3.bandwidth, dtype=np.int64) * U3).astype(np.int32), t3.is_compute)
            ref = [oracle.split_gamma(D3, k3, pu[i], pw[i], pt[i]) for i in range(0, 256, 32)]
            gamma["parity_vs_oracle"] = {"checked_pairs": len(ref), "mismatches": int(sum(int(got[i * 32]) != ref[i] for i in range(len(ref))))}
        g3.close()
        out["split_gamma"] = gamma

        # ---- the generator's back end on a whole topology: Algorithm 2's loop around gamma batches (every switch split
        # off), then spanning tree construction (Appendix E.3) on the switch-free digraph it leaves
        legs = [int(x) for x in args.back_end.split(",") if x.strip() and int(x) != 0]
        if any(x not in (3, 4, 6) for x in legs):
            raise SystemExit("bench.py: --back-end takes 3, 4, 6 (comma-separated) or 0")
        out["back_end"] = []
        for leg in legs:
            tb = w.eulerian_fabric_1024() if leg == 6 else w.config_topology(leg)
            gb = fc.fc_graph_upload(tb.n_vertices, tb.tail, tb.head, tb.bandwidth, tb.is_compute)
            t0 = time.perf_counter()
            sb = fc.fc_opt_throughput_search(gb, 16)
            search_b_ms = (time.perf_counter() - t0) * 1e3
            Ub, kb = sb["U"].numerator, sb["k"] * sb["U"].denominator
            gb.close()
            capb = (np.asarray(tb.bandwidth, dtype=np.int64) * Ub).astype(np.int32)
            t0 = time.perf_counter()
            rs = fc.fc_remove_switches(tb.n_vertices, tb.tail, tb.head, capb, tb.is_compute, kb)
            el_r = time.perf_counter() - t0
            comp_t = np.flatnonzero(np.asarray(tb.is_compute)).tolist()
            idx_t = {v: i for i, v in enumerate(comp_t)}
            links_t = {(idx_t[a], idx_t[b]): c for (a, b), c in rs["links"].items()}
            t0 = time.perf_counter()
            tr = fc.fc_construct_trees(len(comp_t), links_t, kb)
            el_t = time.perf_counter() - t0
            # what the construction promises: out-trees that span, k per root, no link used beyond its capacity
            use_t, per_t, ok_t = {}, {}, True
            for root_t, mult_t, edges_t in tr["trees"]:
                seen_t = {root_t}
                for x_t, y_t in edges_t:
                    ok_t = ok_t and x_t in seen_t and y_t not in seen_t
                    seen_t.add(y_t)
                    use_t[(x_t, y_t)] = use_t.get((x_t, y_t), 0) + mult_t
                ok_t = ok_t and len(seen_t) == len(comp_t)
                per_t[root_t] = per_t.get(root_t, 0) + mult_t
            ok_t = ok_t and per_t == {u: kb for u in range(len(comp_t))} and all(c <= links_t[e] for e, c in use_t.items())
            out["back_end"].append({
                "workload": f"{tb.name} at U = {Ub}, k = {kb}: {len(comp_t)} compute nodes, {tb.n_vertices - len(comp_t)} switches",
                "search_wall_ms": search_b_ms,
                "remove_switches": {"wall_ms": el_r * 1e3, "batches": rs["batches"], "links_out": len(rs["links"]),
                                    "table_entries": sum(len(v) for v in rs["table"].values())},
                "construct_trees": {"wall_ms": el_t * 1e3, "launches": tr["batches"], "root_sets": len(tr["trees"]),
                                    "tree_edges_with_multiplicity": int(sum(m * len(e) for _, m, e in tr["trees"])),
                                    "valid": bool(ok_t)}})
        for _ in range(3):
            H["feas"]()
        torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        import oracle
        flows = H["feas"](want_flows=True)["flows"]
        torch.cuda.synchronize()
        gpu_flows = flows.cpu().numpy().astype(np.int64).reshape(-1)
        pl = H["pl"]
        cores = max(1, min(16, os.cpu_count() or 1))
        # bounded sample: about 20 s of single-core work at ~1.2 ms per solve on the largest config
        stride = max(1, P // 16384)
        idx = np.arange(0, P, stride)
        t0 = time.perf_counter()
        ref = oracle.aux_maxflow_batch(topo, pl.sink[idx], pl.edge_mult[idx], pl.src_cap[idx], threads=cores)
        t_all = time.perf_counter() - t0
        idx1 = idx[:: max(1, len(idx) // 1024)]
        t0 = time.perf_counter()
        oracle.aux_maxflow_batch(topo, pl.sink[idx1], pl.edge_mult[idx1], pl.src_cap[idx1], threads=1)
        t_one = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": len(idx) / t_all, "unit": "solves/s", "cores": cores, "kind": "oracle",
                               "sample": f"{len(idx)} of the step's {P} problems (Dinic, gcc -O2, problems split "
                                         f"statically over {cores} threads)",
                               "single_thread_value": len(idx1) / t_one, "single_thread_sample": len(idx1),
                               "host": {"cpu_model": _cpu_model(), "logical_cpus": os.cpu_count()}}
        batch_flows = H["d_out"].cpu().numpy().astype(np.int64) if entry_point == "fc_maxflow_batch" else gpu_flows
        out["parity_vs_oracle"] = {"checked": int(len(idx)), "mismatches": int((gpu_flows[idx] != ref).sum()),
                                   "mismatches_fc_maxflow_batch": int((batch_flows[idx] != ref).sum())}
    g.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
