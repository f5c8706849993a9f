#!/usr/bin/env python3
"""Benchmark of the DynLP batch-update path on one MI355X.

A *step* is one pass of the whole hot path over one synthetic insertion batch:
dynlp_apply_batch (edge insertion + degree update, seed clamping, frontier seeding, the
frontier-restricted propagation loop to an empty frontier) followed by dynlp_get_labels (argmax).
All inputs are resident in HBM before the timed region (device-pointer mode of the C ABI).

Prints ONE JSON line: metric = inserted undirected edges per second over the timed steps, plus
  "roofline"     algorithmic bytes of the frontier row-update kernel / its device time (HIP events
                 on the launch stream, collected inside the library), against the 8 TB/s HBM peak;
  "cpu_baseline" the CPU oracle (plain C, OpenMP over rows) timed on a bounded sample of the same
                 batch on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
_T0 = time.perf_counter()


def progress(msg: str) -> None:
    """One line per finished phase on stderr (stdout carries only the JSON line)."""
    print(f"[bench {time.perf_counter() - _T0:7.1f} s] {msg}", file=sys.stderr, flush=True)


def counted(n: int, what: str):
    """range(n) that reports on stderr whenever 20 s have passed since its last line."""
    last = time.perf_counter()
    for i in range(n):
        yield i
        if time.perf_counter() - last > 20.0:
            progress(f"{what}: {i + 1}/{n}")
            last = time.perf_counter()


def algorithmic_bytes(rows: int, edges: int, C: int) -> int:
    """Per frontier row of length k: queue entry + row meta (20) + k (col, w) pairs (8k) + k gathered
    neighbour rows (4C each) + own old row and new row (8C).  Summed over rows: edges = sum of k."""
    return 8 * edges + 4 * C * (edges + 2 * rows) + 20 * rows


def compulsory_bytes(rows: int, edges: int, C: int, launches: int, vertices: int) -> int:
    """The same rounds if every needed label row moved once per round instead of once per gather: per launch
    8 * entries + 4C * (distinct neighbours + 2 * rows) + 20 * rows.  The library counts rows and entries per
    round, not distinct neighbours; they are taken as min(entries, vertices) per launch, which is exact for the
    rounds over (nearly) all rows that dominate the timed region and an upper bound otherwise."""
    per_launch_entries = edges / max(1, launches)
    distinct = min(per_launch_entries, float(vertices)) * launches
    return int(8 * edges + 4 * C * (distinct + 2 * rows) + 20 * rows)


def build_workload(name: str, batch_frac: float, num_batches: int, batch_kind: str = "default", scale: float = 1.0):
    import workloads as W

    cfg = W.CONFIGS[name]
    progress(f"generating the base graph of {name}")
    p = W.make_config(name, scale)
    progress(f"base graph: n = {p.n}, {int(p.row_ptr[-1])} entries; generating {num_batches} batches")
    base = dict(n=p.n, C=p.C, row_ptr=p.row_ptr, col=p.col, w=p.w, seed_vertex=p.seed_vertex,
                seed_class=p.seed_class)
    batches = []
    if batch_kind == "clustered":
        # new vertices arriving in groups of similar items (many strong batch-internal edges): the case
        # the component-based label initialisation is for; any base graph
        k = max(1, int(round(batch_frac * cfg["n"])))
        deg = int(cfg.get("batch_degree", cfg.get("mean_degree", cfg.get("k", 10))))
        intra, cross = max(1, deg // 5), max(1, deg // 10)
        for _ in counted(num_batches, 'batches generated'):
            batches.append(W.clustered_batch(p, k, 8.0, intra, cross, max(1, deg - intra - cross),
                                             max(1, int(round(cfg["seed_frac"] * k)))))
        label = (f"{name}: base graph n={cfg['n']} C={cfg['C']}, clustered batches of {k} new vertices "
                 f"(runs of mean length 8; {intra} strong partners in the run, {cross} in the batch, "
                 f"{max(1, deg - intra - cross)} among old vertices)")
    elif cfg["kind"] == "sbm":
        k = max(1, int(round(batch_frac * cfg["n"])))
        for _ in counted(num_batches, 'batches generated'):
            batches.append(W.sbm_vertex_batch(p, k, cfg["batch_degree"], cfg["seed_frac"]))
        label = f"{name}: SBM n={cfg['n']} C={cfg['C']} mean degree {cfg['mean_degree']:g}, batches of {k} new vertices x degree {cfg['batch_degree']}"
    elif cfg["kind"] == "sbm-edge-stream":
        for _ in counted(num_batches, 'batches generated'):
            batches.append(W.sbm_edge_batch(p, cfg["edges_per_batch"], cfg["intra_frac"], cfg["revealed_per_batch"]))
        label = f"{name}: SBM n={cfg['n']} C={cfg['C']}, edge-only batches of {cfg['edges_per_batch']} edges + {cfg['revealed_per_batch']} revealed seeds"
    elif cfg["kind"] == "knn":
        k = max(1, int(round(batch_frac * cfg["n"])))
        for _ in counted(num_batches, 'batches generated'):
            batches.append(W.knn_mixture_batch(p, k, max(1, int(round(cfg["seed_frac"] * k)))))
        label = f"{name}: kNN mixture n={cfg['n']} C={cfg['C']} k={cfg['k']}, batches of {k} new points"
    elif cfg["kind"] == "chung_lu":
        k = max(1, int(round(batch_frac * cfg["n"])))
        for _ in counted(num_batches, 'batches generated'):
            batches.append(W.chung_lu_vertex_batch(p, k, cfg["seed_frac"]))
        label = f"{name}: Chung-Lu n={cfg['n']} C={cfg['C']} mean degree {cfg['mean_degree']:g}, batches of {k} new vertices"
    elif cfg["kind"] == "er-single-batch":
        b = p.state["single_batch"]
        batches = [b] * num_batches  # every step starts from a fresh context holding only the labelled vertices
        label = (f"{name}: Erdos-Renyi n={cfg['n']} mean degree {cfg['mean_degree']:g}, binary labels, "
                 f"{p.n} labelled vertices, all {b.num_new_vertices} unlabelled vertices in one batch")
    else:
        raise KeyError(name)
    return cfg, base, batches, label


def cpu_baseline(base, batches_applied, batch, F_before, tol, gpu_edges_traversed, budget_s, F_cold=None, F_after=None):
    """Oracle Step 3 on the host cores for the first rounds of ``batch`` (bounded by budget_s),
    scaled to the metric's unit with the total work the GPU needed for the same batch."""
    from oracle import native as ON
    from oracle import reference as R

    if base["col"].shape[0] > 100_000_000:
        # Rebuilding the updated CSR on the host (a 370M-key sort) would eat the whole budget, so the
        # sample is the oracle's Jacobi sweep (the same weighted-mean row loop Step 3 runs) over the
        # base graph from the labels the GPU held before the batch.
        sc = np.full(base["n"], -1, dtype=np.int32)
        sc[base["seed_vertex"]] = base["seed_class"]
        w64 = base["w"].astype(np.float64)
        F = F_before[:base["n"]].astype(np.float64)
        entries_per_sweep = int(np.diff(base["row_ptr"])[sc < 0].sum())
        residual = None
        if F_cold is not None:  # how far one exact sweep moves the labels the GPU's cold start ended with
            _, residual = ON.itlp_sweep(base["row_ptr"], base["col"], w64, F_cold.astype(np.float64), sc)
        t0 = time.perf_counter()
        F, _ = ON.itlp_sweep(base["row_ptr"], base["col"], w64, F, sc)
        probe = time.perf_counter() - t0
        progress(f"oracle: one sweep of the base graph takes {probe:.2f} s")
        sweeps = int(max(1, min(1000, 0.8 * budget_s / max(probe, 1e-3))))
        t0 = time.perf_counter()
        for _ in range(sweeps):
            F, _ = ON.itlp_sweep(base["row_ptr"], base["col"], w64, F, sc)
        t_used = time.perf_counter() - t0
        edges = sweeps * entries_per_sweep
        edges_per_s = edges / max(t_used, 1e-9)
        est_latency = gpu_edges_traversed / max(edges_per_s, 1e-9)
        return dict(value=batch.num_edges / est_latency, unit="edges/s", cores=ON.num_threads(), kind="oracle",
                    sample=f"oracle ItLP sweeps (float64, C + OpenMP; the row loop of Step 3) over the base graph: {sweeps} "
                           f"sweeps = {edges} CSR entries in {t_used:.2f} s = {edges_per_s / 1e6:.1f} M entries/s; "
                           f"whole-batch latency extrapolated to the {gpu_edges_traversed} entries the full update "
                           f"traverses = {est_latency:.1f} s",
                    traversed_entries_per_s=edges_per_s,
                    oracle_residual=dict(state="GPU labels after the cold start, one float64 sweep over the base graph",
                                         max_change=residual))

    g = R.Graph(base["n"], base["row_ptr"], base["col"], base["w"], base["C"], base["seed_vertex"], base["seed_class"])
    for b in batches_applied:
        g.insert(b.num_new_vertices, b.eu, b.ev, b.ew, b.seed_vertex, b.seed_class)
    n_old = g.n
    g.insert(batch.num_new_vertices, batch.eu, batch.ev, batch.ew, batch.seed_vertex, batch.seed_class)
    rp, col, w = g.csr()
    progress("oracle: graph with the first timed batch built")
    F = np.concatenate([F_before.astype(np.float64), np.full((batch.num_new_vertices, g.C), 1.0 / g.C)])
    s = np.asarray(batch.seed_vertex, dtype=np.int64)
    F[s] = 0
    F[s, np.asarray(batch.seed_class, dtype=np.int64)] = 1
    A0 = ON.affected_set(rp, col, g.seed_class, n_old, batch.eu, batch.ev, batch.seed_vertex)
    # probe two rounds to size the sample, then one run of as many rounds as the budget allows
    t0 = time.perf_counter()
    out = ON.step3_propagate(rp, col, w, F, g.seed_class, A0, tol, 2, record=16)
    probe = time.perf_counter() - t0
    want = int(max(2, min(100000, 0.8 * budget_s / max(probe / 2, 1e-4))))
    t0 = time.perf_counter()
    out = ON.step3_propagate(rp, col, w, F, g.seed_class, A0, tol, want, record=16)
    t_used = time.perf_counter() - t0
    rounds, edges = out["rounds"], out["edges_traversed"]
    edges_per_s = edges / max(t_used, 1e-9)
    est_latency = gpu_edges_traversed / max(edges_per_s, 1e-9)
    return dict(value=batch.num_edges / est_latency, unit="edges/s", cores=ON.num_threads(), kind="oracle",
                sample=f"oracle Step 3 (float64, C + OpenMP) on the first {rounds} rounds of one batch: "
                       f"{edges} CSR entries traversed in {t_used:.2f} s = {edges_per_s / 1e6:.1f} M entries/s; "
                       f"whole-batch latency extrapolated to the {gpu_edges_traversed} entries the full update traverses "
                       f"= {est_latency:.1f} s",
                traversed_entries_per_s=edges_per_s,
                oracle_residual=dict(state="GPU labels after the first timed batch, one float64 sweep over the updated graph",
                                     max_change=(ON.itlp_sweep(rp, col, w, F_after.astype(np.float64), g.seed_class)[1]
                                                 if F_after is not None else None)))


def residual_after(base, applied, F_last, tol, rounds_total):
    """One float64 oracle sweep over the labels the GPU held after the last timed batch, on the updated graph as
    the harness (not the library) builds it from the base graph and every applied batch.  Returns a dict."""
    import workloads as W
    from oracle import native as ON

    t0 = time.perf_counter()
    k = sum(b.num_new_vertices for b in applied)
    allb = W.Batch(num_new_vertices=k, eu=np.concatenate([b.eu for b in applied]),
                   ev=np.concatenate([b.ev for b in applied]), ew=np.concatenate([b.ew for b in applied]),
                   seed_vertex=np.concatenate([b.seed_vertex for b in applied]),
                   seed_class=np.concatenate([b.seed_class for b in applied]))
    rp, col, w = W.csr_with_batch(base["n"], base["row_ptr"], base["col"], base["w"], allb)
    sc = np.full(base["n"] + k, -1, dtype=np.int32)
    sc[base["seed_vertex"]] = base["seed_class"]
    sc[allb.seed_vertex] = allb.seed_class
    t_build = time.perf_counter() - t0
    progress(f"harness-built updated graph ready ({t_build:.1f} s)")
    t0 = time.perf_counter()
    _, res = ON.itlp_sweep(rp, col, w.astype(np.float64), F_last.astype(np.float64), sc)
    t_sweep = time.perf_counter() - t0
    return dict(state=f"GPU labels after the last timed batch ({len(applied)} batches applied), one float64 oracle sweep "
                      f"over the harness-built updated graph ({int(rp[-1])} entries)",
                max_change=res, seconds_graph_build=round(t_build, 1), seconds_sweep=round(t_sweep, 1),
                # what row-by-row stopping allows (Alg. 2 Step 3): each of the batches' rounds may add tol
                implied_by_stop_rule=(rounds_total + len(applied)) * tol + 2e-6)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg6"])
    ap.add_argument("--batch-frac", type=float, default=0.01, help="new vertices per batch as a fraction of n")
    ap.add_argument("--tol", type=float, default=None, help="threshold delta (default: the workload's)")
    ap.add_argument("--group-lanes", type=int, default=0)
    ap.add_argument("--cpu-budget", type=float, default=20.0, help="seconds of CPU oracle work (0 = skip)")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="do not bracket the row-update launches with HIP events (roofline fields become 0)")
    ap.add_argument("--batch-kind", default="default", choices=["default", "clustered"],
                    help="default: the workload's own batch recipe; clustered: new vertices in groups of similar items")
    ap.add_argument("--init", default="uniform", choices=["uniform", "supernode"],
                    help="starting rows of inserted vertices: 1/C, or Alg. 2 Steps 1-2 (components of the sparsified "
                         "batch-internal graph, tau = mean edge weight of the base graph)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload's vertex count (same law)")
    ap.add_argument("--binary-scalar", type=int, default=-1,
                    help="1: one float per vertex (needs C = 2); 0: n x C rows; default: 1 for cfg6, else 0")
    ap.add_argument("--binned-rounds", type=int, default=0,
                    help="scalar labels: 0 = the library decides, -1 = never, 8..15 = always with 2^k receivers per bin")
    ap.add_argument("--delete-frac", type=float, default=0.0,
                    help="also delete this fraction of a batch's vertex count from the existing vertices in every batch "
                         "(the paper's experiments use 9 deletions per 91 insertions: 0.099)")
    ap.add_argument("--update-mode", default="in-place", choices=["synchronous", "in-place"],
                    help="synchronous: every row of a round reads the round-start labels; in-place: rows are "
                         "replaced at once (Alg. 2's parallel loop taken literally)")
    ap.add_argument("--host-inputs", action="store_true",
                    help="hand the library host arrays (PCIe-inclusive timing; not the headline number)")
    ap.add_argument("--pinned-inputs", action="store_true",
                    help="with --host-inputs: keep the host arrays in pinned memory (the pipelined ingest then sends them "
                         "without staging)")
    ap.add_argument("--persistent-rounds", type=int, default=0,
                    help="1: many rounds per launch (a tuning knob for small graphs); 0: one launch per round")
    ap.add_argument("--final-check", action="store_true",
                    help="dynlp_set_final_check: every batch ends with a round over all rows that moves none by more than tol")
    ap.add_argument("--other-mode-steps", type=int, default=1,
                    help="after the timed steps, this many more batches in the OTHER update mode at the workload's tol "
                         "(reported under detail.other_update_mode, not part of the metric; 0 = skip)")
    ap.add_argument("--threshold-steps", type=int, default=2,
                    help="after the timed steps, this many more batches at the paper's threshold delta = 1e-4 (reported "
                         "under detail.delta_1e-4, not part of the metric; 0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (one process, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2604_06596_amd as P

    if not torch.cuda.is_available():
        print("bench.py needs a GPU: libdynlp has no CPU path", file=sys.stderr)
        sys.exit(3)
    if not os.path.exists(P.library_path()):
        P.build()
    dev = torch.device("cuda:0")
    t_gen = time.perf_counter()
    extra = 0 if args.workload == "cfg6" else max(0, args.threshold_steps)
    extra_mode = 0 if args.workload == "cfg6" else max(0, args.other_mode_steps)
    cfg, base, batches, label = build_workload(args.workload, args.batch_frac, args.warmup + args.steps + extra_mode + extra,
                                               args.batch_kind, args.scale)
    mode_batches = batches[args.warmup + args.steps:args.warmup + args.steps + extra_mode]
    extra_batches = batches[args.warmup + args.steps + extra_mode:]
    batches = batches[:args.warmup + args.steps]
    tol = float(args.tol if args.tol is not None else cfg["tol"])
    t_gen = time.perf_counter() - t_gen
    progress(f"workload ready ({t_gen:.1f} s)")

    pinned_keep = []

    def dv(a, dt):
        if args.host_inputs:
            a = np.ascontiguousarray(a)
            if args.pinned_inputs and a.size:
                t = torch.from_numpy(a).pin_memory()
                pinned_keep.append(t)
                return t.numpy()
            return a
        return torch.from_numpy(np.ascontiguousarray(a)).to(dt).to(dev)

    # One plain device-to-device copy of known size (256 MiB), outside the timed region: under
    # rocprofv3 --pmc it is the yardstick that turns FETCH_SIZE / WRITE_SIZE readings into bytes.
    cal_src = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device=dev)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    del_rng = np.random.default_rng(20260406 + 77)
    dels = [del_rng.choice(base["n"], size=int(round(args.delete_frac * b.num_new_vertices)), replace=False).astype(np.int32)
            for b in batches]
    d_dels = [dv(x, torch.int32) for x in dels]
    fresh = cfg["kind"] == "er-single-batch"  # every step: a new context, then the one big batch
    scalar = bool(args.binary_scalar) if args.binary_scalar >= 0 else fresh
    Cs = 1 if scalar else base["C"]  # stored label columns
    dev_batch = {}

    def to_dev(b):
        if id(b) not in dev_batch:
            dev_batch[id(b)] = dict(k=b.num_new_vertices, eu=dv(b.eu, torch.int32), ev=dv(b.ev, torch.int32),
                                    ew=dv(b.ew, torch.float32), sv=dv(b.seed_vertex, torch.int32),
                                    sc=dv(b.seed_class, torch.int32))
        return dev_batch[id(b)]

    d_batches = [to_dev(b) for b in batches]
    tot_v = sum(b.num_new_vertices for b in (batches[:1] if fresh else batches + mode_batches + extra_batches))
    tot_e = sum(b.num_edges for b in (batches[:1] if fresh else batches + mode_batches + extra_batches))
    d_base = [dv(base["row_ptr"], torch.int64), dv(base["col"], torch.int32), dv(base["w"], torch.float32),
              dv(base["seed_vertex"], torch.int32), dv(base["seed_class"], torch.int32)]

    def new_context():
        ctx = P.DynLP(base["n"], d_base[0], d_base[1], d_base[2], base["C"], d_base[3], d_base[4],
                      device_ptrs=not args.host_inputs, reserve_vertices=tot_v + 1024, reserve_edges=2 * tot_e + 1024,
                      time_kernels=not args.no_kernel_timing, group_lanes=args.group_lanes, binary_scalar=scalar,
                      binned_rounds=args.binned_rounds, persistent_rounds=args.persistent_rounds)
        if args.update_mode == "in-place":
            ctx.set_update_mode(P.UPDATE_IN_PLACE)
        ctx.set_final_check(args.final_check)
        st_, s_ = ctx.static_solve(tol, cfg["max_iter"])
        t_ = None
        if args.init == "supernode":
            # the base graph of cfg6 holds labelled vertices only; its mean weight is the data set's law
            t_ = float(np.float32(ctx.mean_edge_weight()))
            ctx.set_initialiser(P.INIT_SUPERNODE, t_)
        return ctx, st_, s_, t_

    d, st, s0, tau = new_context()
    progress(f"cold start: {s0.iterations} sweeps, {s0.ms_total:.1f} ms")
    # what plain streaming kernels sustain on this machine: 1 GiB copy (read + write) and 1 GiB read-only pass
    copy_gbs, read_gbs = d.stream_bandwidth(1 << 30, 10)
    # ... and what random whole-row gathers of this workload's stored row size sustain in a table of its vertex count
    CP_ = next(c for c in (1, 2, 4, 8, 16, 32, 64) if c >= Cs)
    table_rows = max(1, base["n"] + tot_v)  # the vertex count the timed batches work on
    gather_rows_per_s, gather_gbs = d.gather_bandwidth(table_rows, max(16, 4 * CP_),
                                                       min(400_000_000, max(1_000_000, int(base["col"].shape[0]))), 5)
    cold = dict(status=st, sweeps=s0.iterations, ms=s0.ms_total, ms_update_kernel=s0.ms_update_kernel,
                algorithmic_gbs=algorithmic_bytes(s0.rows_updated, s0.edges_traversed, Cs) / 1e6 /
                max(s0.ms_update_kernel, 1e-9))
    init_info = []
    F_before = None
    F_after = None
    big = base["col"].shape[0] > 100_000_000
    F_cold = None
    if args.cpu_budget > 0 and not fresh and big:
        F_cold = d.get_labels(soft=True, hard=False)[0]
        F_cold = F_cold if args.host_inputs else F_cold.cpu().numpy()
    per_step = []
    round_profile = []
    buckets = {}
    rounds_all = 0  # rounds of every batch applied, warm-up included
    for i, b in enumerate(d_batches):
        timed = i >= args.warmup
        if i == args.warmup and args.cpu_budget > 0 and not fresh:
            F_before = d.get_labels(soft=True, hard=False)[0]
            F_before = F_before if args.host_inputs else F_before.cpu().numpy()
        if fresh and i > 0:
            d.destroy()
            d, _, _, tau = new_context()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if len(dels[i]):
            st, s = d.apply_update(d_dels[i], b["k"], b["eu"], b["ev"], b["ew"], b["sv"], b["sc"])
        else:
            st, s = d.apply_batch(b["k"], b["eu"], b["ev"], b["ew"], b["sv"], b["sc"])
        _, hard = d.get_labels(soft=False, hard=True)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        rounds_all += s.iterations
        progress(f"batch {i + 1}/{len(d_batches)} ({'timed' if timed else 'warm-up'}): {dt * 1e3:.1f} ms, {s.iterations} rounds")
        if timed:
            per_step.append(dict(ms=dt * 1e3, status=st, edges=batches[i].num_edges, **s.as_dict()))
            if tau is not None:
                ii = d.last_components(want_comp=False)[1]
                init_info.append(dict(components=int(ii.components), kept_edges=int(ii.kept_edges),
                                      hook_steps=int(ii.hook_steps), ms=round(float(ii.ms), 3)))
            info = d.round_log_full()
            for r in info:  # per kernel instantiation: launches, rows, entries, device ms
                b = buckets.setdefault((int(r.staged), int(r.group_lanes)), [0, 0, 0, 0.0])
                b[0] += 1
                b[1] += int(r.rows_short + r.rows_long)
                b[2] += int(r.entries_short + r.entries_long)
                b[3] += float(r.ms_update)
            if len(per_step) == 1 and args.cpu_budget > 0 and not fresh and not big and args.delete_frac == 0:
                F_after = d.get_labels(soft=True, hard=False)[0]
                F_after = F_after if args.host_inputs else F_after.cpu().numpy()
            if len(per_step) == 1:  # how the row-update kernels behave as V_aff grows and shrinks
                pick = sorted(set(np.linspace(0, len(info) - 1, num=min(16, len(info))).astype(int).tolist()))
                round_profile = [dict(round=int(j), frontier=int(info[j].rows_short + info[j].rows_long),
                                      staged=int(info[j].staged),
                                      kernel_us=round(float(info[j].ms_update) * 1e3, 1)) for j in pick]
    # labels after the last timed batch, for the oracle's residual check
    F_last = None
    if args.cpu_budget > 0 and not fresh and args.delete_frac == 0:
        F_last = d.get_labels(soft=True, hard=False)[0]
        F_last = F_last if args.host_inputs else F_last.cpu().numpy()
    # the same workload in the other update mode (the timed mode is the in-place one unless asked otherwise; the
    # synchronous one is the reproducible one): a batch or two on the same context
    mode_block = None
    if mode_batches:
        other = "synchronous" if args.update_mode == "in-place" else "in-place"
        d.set_update_mode(P.UPDATE_SYNCHRONOUS if other == "synchronous" else P.UPDATE_IN_PLACE)
        ms_, rounds_, kms_ = [], [], []
        for b in mode_batches:
            db = to_dev(b)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            st, s = d.apply_batch(db["k"], db["eu"], db["ev"], db["ew"], db["sv"], db["sc"])
            _, hard = d.get_labels(soft=False, hard=True)
            torch.cuda.synchronize()
            ms_.append(round((time.perf_counter() - t0) * 1e3, 2))
            rounds_.append(s.iterations)
            kms_.append(round(s.ms_update_kernel, 2))
            rounds_all += s.iterations
        progress(f"{len(ms_)} batches in the {other} mode: {ms_} ms")
        mode_block = dict(update_mode=other, batches=len(ms_), ms_per_batch=ms_, rounds=rounds_, ms_update_kernel=kms_,
                          inserted_edges_per_s=sum(b.num_edges for b in mode_batches) / max(1e-9, sum(ms_) / 1e3))
        d.set_update_mode(P.UPDATE_IN_PLACE if args.update_mode == "in-place" else P.UPDATE_SYNCHRONOUS)
    # the paper's own threshold (delta = 1e-4, its "near optimal accuracy" choice): a few more batches on the same
    # context, where V_aff stays a small part of the graph and the flag-marking rounds dominate
    delta_block = None
    if extra_batches:
        d.set_params(1e-4, cfg["max_iter"])
        xs, xb = [], {}
        for b in extra_batches:
            db = to_dev(b)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            st, s = d.apply_batch(db["k"], db["eu"], db["ev"], db["ew"], db["sv"], db["sc"])
            _, hard = d.get_labels(soft=False, hard=True)
            torch.cuda.synchronize()
            xs.append(dict(ms=(time.perf_counter() - t0) * 1e3, status=st, edges=b.num_edges, **s.as_dict()))
            for r in d.round_log_full():
                q = xb.setdefault((int(r.staged), int(r.group_lanes)), [0, 0, 0, 0.0])
                q[0] += 1
                q[1] += int(r.rows_short + r.rows_long)
                q[2] += int(r.entries_short + r.entries_long)
                q[3] += float(r.ms_update)
        progress(f"{len(xs)} batches at delta = 1e-4: {[round(x['ms'], 1) for x in xs]} ms")
        CPx = next(c for c in (1, 2, 4, 8, 16, 32, 64) if c >= Cs)
        kx = {}
        for (staged, glanes), (cnt, rws, ent, ms) in xb.items():
            name = ("k_pb_scatter + k_pb_gather" if staged == 3 else f"k_row_update_pull<{CPx}, {glanes}>" if staged == 2 else
                    f"k_row_update<{CPx}, {glanes}, {'true' if staged else 'false'}>")
            kx[name] = dict(launches=cnt, rows=rws, entries=ent, device_ms=round(ms, 3), avg_launch_us=round(ms * 1e3 / max(1, cnt), 1),
                            algorithmic_GBs=round(algorithmic_bytes(rws, ent, Cs) / 1e6 / max(ms, 1e-9), 1))
        delta_block = dict(tol=1e-4, batches=len(xs), ms_per_batch=[round(x["ms"], 2) for x in xs],
                           inserted_edges_per_s=sum(x["edges"] for x in xs) / max(1e-9, sum(x["ms"] for x in xs) / 1e3),
                           rounds=[x["iterations"] for x in xs], frontier_initial=[x["frontier_initial"] for x in xs],
                           frontier_peak=[x["frontier_peak"] for x in xs],
                           ms_insert=[round(x["ms_insert"], 3) for x in xs], ms_seed=[round(x["ms_seed"], 3) for x in xs],
                           ms_iterate=[round(x["ms_iterate"], 3) for x in xs],
                           ms_update_kernel=[round(x["ms_update_kernel"], 3) for x in xs], row_update_kernels=kx,
                           note="same context after the timed batches; labels were converged at the workload's tol before")
        d.set_params(tol, cfg["max_iter"])
    total_s = sum(x["ms"] for x in per_step) / 1e3
    edges_inserted = sum(x["edges"] for x in per_step)
    rows = sum(x["rows_updated"] for x in per_step)
    trav = sum(x["edges_traversed"] for x in per_step)
    # The roofline entry is for the kernel that takes the most device time in the timed region.
    CP = next(c for c in (1, 2, 4, 8, 16, 32, 64) if c >= Cs)
    kstats = {}
    for (staged, glanes), (cnt, rws, ent, ms) in buckets.items():
        name = ("k_pb_scatter + k_pb_gather" if staged == 3 else f"k_row_update_pull<{CP}, {glanes}>" if staged == 2 else
                f"k_row_update<{CP}, {glanes}, {'true' if staged else 'false'}>")
        ab = algorithmic_bytes(rws, ent, Cs)
        kstats[name] = dict(launches=cnt, rows=rws, entries=ent, device_ms=round(ms, 3),
                            avg_launch_us=round(ms * 1e3 / max(1, cnt), 1),
                            algorithmic_GBs=round(ab / 1e6 / max(ms, 1e-9), 1), algorithmic_bytes=ab)
    dom = max(kstats, key=lambda k: kstats[k]["device_ms"])
    launches = kstats[dom]["launches"]
    k_ms = kstats[dom]["device_ms"]
    alg_bytes = kstats[dom]["algorithmic_bytes"]
    achieved = alg_bytes / 1e6 / max(k_ms, 1e-9)  # GB/s
    all_ms = sum(v["device_ms"] for v in kstats.values())
    all_bytes = sum(v["algorithmic_bytes"] for v in kstats.values())
    # HBM-side bytes per launch by the counters: profiles/ stores, per kernel, the ratio of counter bytes (rocprofv3
    # --pmc, request-size counters) to algorithmic bytes over a whole profiling run of the same workload; applied
    # here to this run's algorithmic bytes per launch, so that the two figures describe the same rows and entries.
    traffic = None
    traffic_ratio = None
    tpath = os.path.join(ROOT, "profiles", f"row_update_{args.workload}_hbm_traffic.md")
    if os.path.exists(tpath):
        import re
        for hit in re.finditer(r"hbm_bytes_per_algorithmic_byte = ([0-9.]+) for kernel `([^`]+)`", open(tpath).read()):
            if hit.group(2).endswith(dom):
                traffic_ratio = float(hit.group(1))
                traffic = traffic_ratio * alg_bytes / max(1, launches)
    comp_bytes = compulsory_bytes(kstats[dom]["rows"], kstats[dom]["entries"], Cs, launches, d.num_vertices)
    out = {
        "metric": "dynlp_batch_update_inserted_edges_per_s",
        "value": edges_inserted / total_s,
        "unit": "edges/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": total_s * 1e3 / max(1, len(per_step)),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic" + ((" (host-resident inputs, " + ("pinned" if args.pinned_inputs else "pageable") +
                                ": PCIe-inclusive)") if args.host_inputs else ""),
        "config": {"workload": label, "tol": tol, "update_mode": args.update_mode, "binary_scalar": scalar, "edges_per_batch": edges_inserted // max(1, len(per_step)),
                   "vertices_after": d.num_vertices, "directed_entries_after": d.num_entries},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": dom, "launches": launches,
                     "avg_launch_us": k_ms * 1e3 / max(1, launches),
                     "algorithmic_bytes_per_launch": alg_bytes / max(1, launches),
                     # what the counters say the same launch moves on the HBM side, as a rate (context: `frac`
                     # above is the algorithmic one)
                     "stream_copy_GBs": copy_gbs, "stream_read_GBs": read_gbs, "frac_of_stream_read": achieved / read_gbs,
                     # gathers per second: this kernel's CSR entries per second against random whole-row reads of the
                     # same stored row size with no other traffic
                     "gather_yardstick": {"row_bytes": max(16, 4 * CP_), "table_rows": table_rows,
                                          "rows_per_s": gather_rows_per_s, "GBs": gather_gbs},
                     "gathers_per_s": kstats[dom]["entries"] / max(k_ms * 1e-3, 1e-12),
                     "frac_of_gather_yardstick": kstats[dom]["entries"] / max(k_ms * 1e-3, 1e-12) / max(gather_rows_per_s, 1.0),
                     "traffic_per_algorithmic_byte": traffic_ratio,
                     "traffic_GBs": (traffic / (k_ms * 1e6 / max(1, launches))) if traffic and k_ms > 0 else None,
                     "compulsory_bytes_per_launch": comp_bytes / max(1, launches),
                     "compulsory_GBs": comp_bytes / 1e6 / max(k_ms, 1e-9)},
        "detail": {"rounds_per_step": [x["iterations"] for x in per_step],
                   "frontier_initial": [x["frontier_initial"] for x in per_step],
                   "frontier_peak": [x["frontier_peak"] for x in per_step],
                   "traversed_entries_per_s": trav / total_s,
                   "ms_insert": [round(x["ms_insert"], 3) for x in per_step],
                   "ms_seed": [round(x["ms_seed"], 3) for x in per_step],
                   "ms_iterate": [round(x["ms_iterate"], 3) for x in per_step],
                   "ms_update_kernel": [round(x["ms_update_kernel"], 3) for x in per_step],
                   "status": [x["status"] for x in per_step],
                   "row_update_kernels": {k: {kk: vv for kk, vv in v.items() if kk != "algorithmic_bytes"}
                                          for k, v in kstats.items()},
                   "row_update_all_kernels_algorithmic_GBs": round(all_bytes / 1e6 / max(all_ms, 1e-9), 1),
                   "round_profile_first_step": round_profile,
                   "cold_start": cold, "gen_s": round(t_gen, 1),
                   "init": {"mode": args.init, "tau": tau, "per_step": init_info},
                   "update_mode": args.update_mode, "final_check": bool(args.final_check),
                   "final_checks_per_step": [x["final_checks"] for x in per_step],
                   "ingest_chunks_per_step": [x["ingest_chunks"] for x in per_step],
                   "other_update_mode": mode_block,
                   "delta_1e-4": delta_block,
                   "deleted_per_step": [int(len(x)) for x in dels[args.warmup:]]},
    }
    if args.cpu_budget > 0 and per_step and not fresh:
        progress("CPU oracle baseline")
        out["cpu_baseline"] = cpu_baseline(base, batches[:args.warmup], batches[args.warmup], F_before, tol,
                                           per_step[0]["edges_traversed"], args.cpu_budget, F_cold=F_cold, F_after=F_after)
    else:
        out["cpu_baseline"] = None
    if out["cpu_baseline"] is not None and F_last is not None:
        progress("oracle sweep over the labels after the last batch")
        out["cpu_baseline"]["oracle_residual_after_last_batch"] = residual_after(
            base, batches, F_last, tol, rounds_all)
    d.destroy()
    progress("done")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
