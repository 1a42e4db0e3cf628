"""Benchmark of the batched variant-selection path on one MI355X.

One "step" is one call of infaas_sel_select over the whole query batch of the chosen
configuration (default: configuration 2 -- 50 tasks x 2,000 variants, 16M queries with Zipf
task popularity), inputs already resident in HBM.  For the streaming configuration (4) a step
is one 4M-query chunk preceded by its load update (10% of the variants).

With --closest a step is one call of infaas_sel_select_closest (the selection plus a suggestion
for the queries that nothing satisfies; 24 B per decision).  With --tiered a step is one call of
infaas_sel_select_tiered over seeded variant states (Active variants first, else an Inactive one
by loading + inference latency; variant and tier arrays, 24 B per decision); its two lookup
launches are priced together.  With --workers a step is one call of infaas_sel_select_workers
(the same plus the worker that serves each answer, over a seeded cluster; 28 B per decision).
With --getvariant a step is one call of infaas_sel_select_workers_closest (that plus the closest
variant where neither tier answers; 32 B per decision).
With --scale a step is one call of infaas_sel_scale over 4M seeded scaling requests on the table of
the configuration (replicate or upgrade on a change in load; 32 B per decision), with --scale-down
one call of infaas_sel_scale_down (keep, remove an instance or downgrade).

Prints ONE JSON line: decisions/s, the roofline of the dominant kernel (algorithmic bytes:
20 B per decision + the variant table once, against 8 TB/s of HBM) timed with HIP events on
the launch stream, and the CPU oracle timed on a bounded sample of the same queries.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
BYTES_PER_DECISION = 20          # 4 int32 query fields read + 1 int32 result written
UPDATE_BYTES = 8                 # one (row, value) pair of a load report
ROTATE_BYTES = 1_400_000_000     # bytes touched between two uses of one buffer (last-level cache: 256 MB)
MAX_SETS = 64                    # (tiny configurations cannot reach ROTATE_BYTES with a sensible number of buffers)
MAX_DISTINCT = 18                # batches drawn from seeds of their own; sets beyond them are device copies


def table_bytes(tb) -> int:
    """Variant store, counted once per call: accuracy, queue and row of every variant plus its
    latency and cost at every batch size (12 + 8 B bytes per variant)."""
    return tb.V * (12 + 8 * tb.B)


def kernel_source_digest() -> str:
    """Digest of the HIP sources; counter readings are only valid for the code they were taken on."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_1905_13348_amd", "csrc", "*"))):
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(kernel: str, cfg: int, engine: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc readings
    (profiles/traffic.json), or None when there are none for this workload or the kernels have
    changed since they were taken."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    if rec.get("source_digest") != kernel_source_digest():
        return None
    return rec.get("bytes_per_launch", {}).get(f"config{cfg}/{engine}/{kernel}")


SCALE_REQUESTS = 4_000_000
SCALE_LAMBDA, SCALE_SLACK = 50, 105
SCALE_BYTES_PER_DECISION = 32    # 5 int32 request fields read + 3 int32 results written


def bench_scale(args, cfg, spec, tb, down=False) -> int:
    """A scaling-decision call (Section 4.2.2: scaling up, or with down=True scaling down) timed like
    the selection."""
    import numpy as np
    import torch

    import paper_1905_13348_amd as pkg
    import workloads

    if args.closest or args.tiered or args.workers or args.case1 or args.getvariant or args.engine != "auto":
        print("bench.py: --scale and --scale-down go alone", file=sys.stderr)
        return 2
    n = min(SCALE_REQUESTS, spec["num_queries"])
    sc = workloads.make_scaling(cfg, tb)
    sel = pkg.Selector(tb.num_tasks, tb.batch_sizes, device=0, engine=pkg.ENGINE_AUTO)
    sel.load_variants(tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    sel.load_scaling(sc.arch_id, sc.sat_qps, sc.hw_cost, sc.load_us, SCALE_LAMBDA, SCALE_SLACK)
    n_sets = int(min(MAX_SETS, max(4, -(-ROTATE_BYTES // (n * SCALE_BYTES_PER_DECISION)))))   # see main()
    make = workloads.make_scale_down_requests if down else workloads.make_scale_requests
    host = [make(cfg, tb, sc, n, chunk=c) for c in range(n_sets)]
    dev = [[torch.from_numpy(x).cuda() for x in (r.variant, r.instances, r.load_qps, r.slo_us, r.batch_idx)]
           for r in host]
    out_sets = [[torch.empty(n, dtype=torch.int32, device="cuda") for _ in range(3)] for _ in range(n_sets)]
    done = 0
    t_heat = time.perf_counter()
    while args.preheat_ms > 0 and 1e3 * (time.perf_counter() - t_heat) < args.preheat_ms:
        for _ in range(16):
            sel.scale(*dev[done % n_sets], *out_sets[done % n_sets], down=down)
            done += 1
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        sel.scale(*dev[done % n_sets], *out_sets[done % n_sets], down=down)
        done += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):   # the timed region, instrumentation off
        sel.scale(*dev[done % n_sets], *out_sets[done % n_sets], down=down)
        done += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    sel.set_timing(True)          # the same steps again for the kernel's own duration
    torch.cuda.synchronize()
    for _ in range(args.steps):
        sel.scale(*dev[done % n_sets], *out_sets[done % n_sets], down=down)
        done += 1
    torch.cuda.synchronize()
    timings = sel.get_timings()
    sel.set_timing(False)
    outs = out_sets[(done - 1) % n_sets]
    ms_per_step = 1e3 * elapsed / args.steps
    kernel = "scale_down" if down else "scale"
    k = timings[kernel]
    avg_ms = k["total_ms"] / k["launches"]
    # every request in, every result out, and what the decision reads of the table once: per variant
    # its architecture, throughput, hardware cost, loading latency and the latency at every batch size
    fixed = tb.V * (16 + 4 * tb.B)
    algo = SCALE_BYTES_PER_DECISION * n + fixed
    achieved = algo / (avg_ms * 1e-3) / 1e9
    cpu, mismatches = None, None
    if not args.no_cpu_baseline:
        import oracle
        ref = oracle.load_oracle()
        rq = host[(done - 1) % n_sets]
        fields = (rq.variant, rq.instances, rq.load_qps, rq.slo_us, rq.batch_idx)
        prof = (sc.arch_id, sc.sat_qps, sc.hw_cost, sc.load_us, tb.lat_us, SCALE_LAMBDA, SCALE_SLACK)
        n0 = min(n, 20_000)
        s0 = time.perf_counter()
        ref.scale(*prof, *(f[:n0] for f in fields), down=down)
        rate0 = n0 / (time.perf_counter() - s0)
        m = int(min(n, max(n0, rate0 * args.cpu_seconds)))
        s0 = time.perf_counter()
        want = ref.scale(*prof, *(f[:m] for f in fields), down=down)
        dt = time.perf_counter() - s0
        mismatches = int(sum((g[:m].cpu().numpy() != w).sum() for g, w in zip(outs, want)))
        cpu = {"value": round(m / dt, 1), "unit": "decisions/s", "cores": ref.num_threads(), "kind": "oracle",
               "sample": f"first {m} requests of the last timed batch, {dt:.1f} s"}
    line = {
        "metric": "variant-selection decisions/sec on 1 MI355X; % of HBM roofline",
        "value": round(n * args.steps / elapsed, 1), "unit": "decisions/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
        "config": {"workload": f"scaling decisions ({'keep, remove an instance or downgrade at the regular check' if down else 'replicate or upgrade on a change in load'}): {n} requests per step on "
                               f"the table of config {cfg} ({tb.V} variants in {int(np.unique(sc.arch_id).size)} "
                               f"architectures, {tb.B} batch sizes), lambda {SCALE_LAMBDA}/s, headroom {SCALE_SLACK}%",
                   "engine": "auto"},
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5),
                     "traffic": measured_traffic(kernel, cfg, "auto/" + kernel), "avg_kernel_ms": round(avg_ms, 5),
                     "algorithmic_bytes_per_launch": int(algo)},
        "kernels_ms_per_step": {kernel: round(k["total_ms"] / args.steps, 5)},
        "cpu_baseline": cpu,
        "parity_sample_mismatches": mismatches,
    }
    print(json.dumps(line))
    sel.destroy()
    return 0 if not mismatches else 1


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (defaults: a GPU that has been idle runs its first 15-20 ms of work -- some 250 steps of the default
    # configuration -- about 7% slower than it does from then on; a serving system is never idle, so the
    # default warm-up is long enough to time the steady state)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--preheat-ms", type=float, default=30.0,
                    help="before the warm-up steps: the same steps, untimed, for at least this long, so that the "
                         "steady state is timed whatever --warmup says (0: none)")
    ap.add_argument("--config", type=int, default=2, choices=[0, 1, 2, 3, 4])
    ap.add_argument("--engine", default="auto", choices=["auto", "scan", "index"])
    ap.add_argument("--table", default="config", choices=["config", "long_staircases", "wide_accuracy"],
                    help="the configuration's own table, or the same table bent into a shape the staircase index "
                         "cannot hold (every variant a possible answer; accuracies beyond its 16-bit keys)")
    ap.add_argument("--degrade", action="store_true",
                    help="before the steps, one load report over all rows that makes every variant a possible answer "
                         "(queues that fall with the cost): the index built at load time no longer fits")
    ap.add_argument("--closest", action="store_true",
                    help="time infaas_sel_select_closest (selection plus a suggestion where nothing is "
                         "feasible; 24 B per decision) instead of infaas_sel_select")
    ap.add_argument("--tiered", action="store_true",
                    help="time infaas_sel_select_tiered (state-aware two-tier selection over seeded variant "
                         "states; 24 B per decision) instead of infaas_sel_select")
    ap.add_argument("--case1", action="store_true",
                    help="time infaas_sel_select_tiered_closest (the complete Case I: two-tier selection plus the "
                         "closest Active or Inactive variant where neither tier answers; 28 B per decision)")
    ap.add_argument("--workers", action="store_true",
                    help="time infaas_sel_select_workers (two-tier selection plus the worker of every answer, "
                         "over a seeded cluster of workers and instances; 28 B per decision)")
    ap.add_argument("--getvariant", action="store_true",
                    help="time infaas_sel_select_workers_closest (the whole of Case I: variant, tier, worker and, where "
                         "neither tier answers, the closest variant; 32 B per decision)")
    ap.add_argument("--scale", action="store_true",
                    help="time infaas_sel_scale (scaling decisions on a change in load: 4M seeded requests, "
                         "lambda 50/s, headroom 105%%; 32 B per decision) instead of the selection")
    ap.add_argument("--scale-down", action="store_true",
                    help="time infaas_sel_scale_down (the regular scaling-down check: keep, remove an instance "
                         "or downgrade; 4M seeded requests, same profile and 32 B per decision)")
    ap.add_argument("--graph", action="store_true",
                    help="after the timed steps (which give the kernel times), capture the steps into HIP graphs "
                         "and time the same number of steps again as graph replays: value and ms_per_step are "
                         "then those of the replays")
    ap.add_argument("--streams", type=int, default=1,
                    help="after the timed steps (which give the kernel times), time the same number of steps again "
                         "dealt in turn to this many streams, each with a handle of its own on the same table (handles "
                         "share nothing, so their calls need no ordering): value and ms_per_step are then those of "
                         "that loop.  Plain selection on a configuration without load reports only.")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device-to-device copy of 256 MiB a few times (reference for "
                         "scaling the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU; queries would shard across GPUs with no "
              "exchange step, but no multi-GPU path exists here. Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_1905_13348_amd as pkg
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate_copy:
        # eight 256 MiB source / destination pairs taken in turn: 4 GiB pass between two uses of
        # the same buffer, so that no copy finds its data in a cache
        pairs = [(torch.arange(64 * 1024 * 1024, dtype=torch.int32, device="cuda") + k,
                  torch.empty(64 * 1024 * 1024, dtype=torch.int32, device="cuda")) for k in range(8)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for r in range(16):
            src, dst = pairs[r % len(pairs)]
            dst.copy_(src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 16
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4,
                          "copies": 16, "pairs": len(pairs), "ms_per_copy_wall": round(1e3 * dt, 4)}))
        return 0
    cfg = args.config
    spec = workloads.config_spec(cfg)
    tb = workloads.make_table(cfg) if args.table == "config" else workloads.make_cliff_table(args.table, cfg)
    if args.scale or args.scale_down:
        if args.scale and args.scale_down:
            print("bench.py: --scale or --scale-down, not both", file=sys.stderr)
            return 2
        return bench_scale(args, cfg, spec, tb, down=args.scale_down)
    chunks = spec["chunks"]
    per_step = spec["num_queries"] // chunks
    engine = {"auto": pkg.ENGINE_AUTO, "scan": pkg.ENGINE_SCAN, "index": pkg.ENGINE_INDEX}[args.engine]
    if (args.closest or args.tiered or args.workers or args.case1 or args.getvariant) and \
            (args.engine != "auto" or args.closest + args.tiered + args.workers + args.case1 + args.getvariant > 1):
        print("bench.py: --closest, --tiered, --case1, --workers and --getvariant need the index engine (--engine auto), "
              "one at a time", file=sys.stderr)
        return 2
    with_cluster = args.workers or args.getvariant

    sel = pkg.Selector(tb.num_tasks, tb.batch_sizes, device=0, engine=engine)
    sel.load_variants(tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    sel.reserve(per_step)
    base_queue = tb.queue_us
    if args.degrade:
        worst = workloads.make_degrading_load_update(tb)
        sel.update_load(torch.from_numpy(worst.variant_idx).cuda(), torch.from_numpy(worst.queue_us).cuda())
        base_queue = worst.queue_us.copy()      # (the report covers every row)
        torch.cuda.synchronize()
    states = None
    cluster = None
    if args.tiered or with_cluster or args.case1:
        states = workloads.make_states(cfg, tb.V)
        sel.load_states(states.state, states.load_us)
    if with_cluster:
        cluster = workloads.make_workers(cfg, states)
        sel.load_workers(cluster.worker_hw, cluster.worker_util, cluster.variant_hw, cluster.inst_variant,
                         cluster.inst_worker, cluster.inst_load)

    # Inputs resident in HBM before the timed region.  The steps rotate over n_sets distinct query
    # batches (different seeds; the streaming configuration: consecutive chunks, each with its load
    # report) and as many result arrays, enough that at least ROTATE_BYTES are touched between two
    # uses of the same buffer: nothing a step reads or writes can still sit in a cache (the part has
    # 256 MB of last-level cache) from the step that used it before.
    two_results = args.closest or args.tiered or with_cluster or args.case1       # suggestion, or tier
    three_results = with_cluster or args.case1                                     # worker, or suggestion beside the tier
    four_results = args.getvariant                                                 # worker and suggestion
    per_decision = BYTES_PER_DECISION + (4 if two_results else 0) + (4 if three_results else 0) + (4 if four_results else 0)
    set_bytes = per_step * per_decision
    n_sets = int(min(MAX_SETS, max(4, -(-ROTATE_BYTES // set_bytes))))
    if chunks > 1:
        n_sets = min(n_sets, chunks)
    if args.streams > 1:
        if chunks > 1 or two_results or args.graph or args.degrade or not 2 <= args.streams <= 4:
            print("bench.py: --streams 2..4 goes with the plain selection on a configuration without load reports",
                  file=sys.stderr)
            return 2
        n_sets += (-n_sets) % args.streams     # a set of buffers is always used on the same stream
    n_distinct = min(n_sets, MAX_DISTINCT)
    host_q = [workloads.make_queries(cfg, chunk=c) for c in range(n_distinct)]
    dev_q = []
    for c in range(n_sets):   # beyond MAX_DISTINCT seeds: device copies (other addresses, same values)
        src = host_q[c % n_distinct]
        dev_q.append([torch.from_numpy(x).cuda() for x in (src.task, src.slo_us, src.min_acc_bp, src.batch_idx)])
    outs = [torch.empty(per_step, dtype=torch.int32, device="cuda") for _ in range(n_sets)]
    seconds = [torch.empty(per_step, dtype=torch.int32, device="cuda") if two_results else None for _ in range(n_sets)]
    workers_out = [torch.empty(per_step, dtype=torch.int32, device="cuda") if three_results else None
                   for _ in range(n_sets)]
    fourths = [torch.empty(per_step, dtype=torch.int32, device="cuda") if four_results else None for _ in range(n_sets)]
    updates = []
    worker_updates = []
    if chunks > 1 and with_cluster:   # a report of the cluster before every step as well
        for c in range(1, n_sets + 1):
            wu = workloads.make_worker_update(cfg, cluster.W, cluster.I, c)
            worker_updates.append(([torch.from_numpy(x).cuda() for x in
                                    (wu.worker_idx, wu.worker_util, wu.inst_idx, wu.inst_load)], wu))
    if chunks > 1:
        for c in range(1, n_sets + 1):
            up = workloads.make_load_update(cfg, tb.V, c)
            updates.append((torch.from_numpy(up.variant_idx).cuda(), torch.from_numpy(up.queue_us).cuda(), up))

    def step(i: int) -> None:
        k = i % n_sets
        if updates:
            u = updates[i % len(updates)]
            sel.update_load(u[0], u[1])
        if args.closest:
            sel.select_closest(*dev_q[k], outs[k], seconds[k])
        elif args.tiered:
            sel.select_tiered(*dev_q[k], outs[k], seconds[k])
        elif args.case1:
            sel.select_tiered_closest(*dev_q[k], outs[k], seconds[k], workers_out[k])
        elif with_cluster:
            if worker_updates:
                sel.update_workers(*worker_updates[i % len(worker_updates)][0])
            if args.getvariant:
                sel.select_workers_closest(*dev_q[k], outs[k], seconds[k], workers_out[k], fourths[k])
            else:
                sel.select_workers(*dev_q[k], outs[k], seconds[k], workers_out[k])
        else:
            sel.select(*dev_q[k], outs[k])

    done = 0      # steps enqueued so far (the load reports of the streaming configuration follow it)
    t_heat = time.perf_counter()
    while args.preheat_ms > 0 and 1e3 * (time.perf_counter() - t_heat) < args.preheat_ms:
        for _ in range(16):
            step(done)
            done += 1
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step(done)
        done += 1
    # 1. the timed region: exactly args.steps steps, library instrumentation off
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(done)
        done += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # 2. the same steps once more with an event pair attached to every kernel launch: per-kernel
    #    durations for the roofline (not part of value / ms_per_step)
    sel.set_timing(True)
    torch.cuda.synchronize()
    for _ in range(args.steps):
        step(done)
        done += 1
    torch.cuda.synchronize()
    timings = sel.get_timings()
    sel.set_timing(False)
    if args.graph:
        # and as graph replays, continuing the sequence of load reports
        period = n_sets
        graphs = []
        for j in range(period):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(j)
            graphs.append(g)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graphs[done % period].replay()
            done += 1
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    if args.streams > 1:
        sels = [sel]
        for _ in range(args.streams - 1):
            other = pkg.Selector(tb.num_tasks, tb.batch_sizes, device=0, engine=engine)
            other.load_variants(tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
            other.reserve(per_step)
            sels.append(other)
        lanes = [torch.cuda.Stream() for _ in sels]
        done += (-done) % n_sets                # step i: buffers i % n_sets, stream and handle i % streams

        def run(count: int) -> None:
            nonlocal done
            for _ in range(count):
                k, j = done % n_sets, done % len(sels)
                with torch.cuda.stream(lanes[j]):
                    sels[j].select(*dev_q[k], outs[k])
                done += 1

        torch.cuda.synchronize()
        run(max(args.warmup, 4 * len(sels)))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(args.steps)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        for other in sels[1:]:
            other.destroy()
    last = done - 1
    ms_per_step = 1e3 * elapsed / args.steps
    value = per_step * args.steps / elapsed

    # ---- roofline of the dominant kernel
    active = {k: v for k, v in timings.items() if v["launches"] > 0}
    dom = max(active, key=lambda k: active[k]["total_ms"])
    dom_avg_ms = active[dom]["total_ms"] / active[dom]["launches"]
    launches_per_step = active[dom]["launches"] / args.steps
    mode = "/closest" if args.closest else "/tiered" if args.tiered else "/workers" if args.workers else \
        "/case1" if args.case1 else "/getvariant" if args.getvariant else ""
    fixed_bytes = table_bytes(tb) + (8 * tb.V if args.tiered or with_cluster or args.case1 else 0)   # + state and loading latency
    if with_cluster:   # + hardware of every variant, the workers, the instances
        fixed_bytes += 4 * tb.V + 8 * cluster.W + 12 * cluster.I
    if dom.startswith("group_"):
        # the group-by-group path is three kernels that only together answer a query: they are
        # priced as one launch, the bytes of the whole call against the sum of their durations
        algo_bytes = per_decision * per_step + fixed_bytes
        dom_avg_ms = sum(active[k]["total_ms"] for k in active if k.startswith("group_")) / args.steps
        dom = "group_bin+group_lookup+group_finish"
    elif (args.tiered or with_cluster or args.case1) and dom == "index_select":
        # one lookup per tier: the pair is priced as one launch against the bytes of the whole call
        algo_bytes = per_decision * per_step + fixed_bytes
        dom_avg_ms = active[dom]["total_ms"] / args.steps
    elif dom == "index_build":     # reads the rank-ordered accuracy and latency+queue columns once
        algo_bytes = 8 * tb.B * tb.V
    elif dom == "update_load":
        algo_bytes = UPDATE_BYTES * updates[0][2].variant_idx.size
    else:                        # a select kernel: every query in, every result out, the table once
        algo_bytes = (per_decision * per_step + fixed_bytes) / launches_per_step
    achieved = algo_bytes / (dom_avg_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 5),
                "traffic": measured_traffic(dom, cfg, args.engine + mode),
                "avg_kernel_ms": round(dom_avg_ms, 5),
                "algorithmic_bytes_per_launch": int(algo_bytes)}
    whole_bytes = per_decision * per_step + fixed_bytes + \
        (UPDATE_BYTES * updates[0][2].variant_idx.size if updates else 0)
    whole_frac = whole_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS

    # ---- the last step's result, checked on a sample, and the oracle timed beside it
    cpu = None
    mismatches = None
    if not args.no_cpu_baseline:
        import oracle
        ref = oracle.load_oracle()
        q = host_q[(last % n_sets) % n_distinct]
        out, closest, worker = outs[last % n_sets], seconds[last % n_sets], workers_out[last % n_sets]
        fourth = fourths[last % n_sets]
        queue = base_queue.copy()
        if updates:  # replay the load reports in the order the steps applied them
            for i in range(last + 1):
                up = updates[i % len(updates)][2]
                ref.update_load(queue, up.variant_idx, up.queue_us)
        fields = (q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
        n0 = min(per_step, 100_000)
        s0 = time.perf_counter()
        if with_cluster:
            util, iload = cluster.worker_util.copy(), cluster.inst_load.copy()
            if worker_updates:
                for i in range(last + 1):
                    wu = worker_updates[i % len(worker_updates)][1]
                    ref.update_worker_util(util, wu.worker_idx, wu.worker_util)
                    ref.update_instance_load(iload, wu.inst_idx, wu.inst_load)

            def ref_fn(*a):
                fn = ref.get_variant if args.getvariant else ref.select_workers
                return fn(*a[:5], states.state, states.load_us, cluster.variant_hw, cluster.worker_hw,
                          util, cluster.inst_variant, cluster.inst_worker, iload, *a[5:])
        elif args.tiered:
            def ref_fn(*a):
                return ref.select_tiered(*a[:5], states.state, states.load_us, *a[5:])
        elif args.case1:
            def ref_fn(*a):
                return ref.select_case1(*a[:5], states.state, states.load_us, *a[5:])
        else:
            ref_fn = ref.select_closest if args.closest else ref.select
        ref_fn(tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, queue, *(f[:n0] for f in fields))
        rate0 = n0 / (time.perf_counter() - s0)
        n = int(min(per_step, max(n0, rate0 * args.cpu_seconds)))
        s0 = time.perf_counter()
        want = ref_fn(tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, queue, *(f[:n] for f in fields))
        dt = time.perf_counter() - s0
        if four_results:
            mismatches = int(sum((g[:n].cpu().numpy() != w).sum() for g, w in zip((out, closest, worker, fourth), want)))
        elif three_results:
            mismatches = int(sum((g[:n].cpu().numpy() != w).sum() for g, w in zip((out, closest, worker), want)))
        elif two_results:
            mismatches = int((out[:n].cpu().numpy() != want[0]).sum() + (closest[:n].cpu().numpy() != want[1]).sum())
        else:
            mismatches = int((out[:n].cpu().numpy() != want).sum())
        cpu = {"value": round(n / dt, 1), "unit": "decisions/s", "cores": ref.num_threads(),
               "kind": "oracle", "sample": f"first {n} queries of the last timed batch, {dt:.1f} s"}
        # and on one host thread, on a sample of about two seconds
        threads = ref.num_threads()
        n1 = int(min(n, max(1000, 2.0 * (n / dt) / max(threads, 1))))
        ref.set_threads(1)
        s0 = time.perf_counter()
        ref_fn(tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, queue, *(f[:n1] for f in fields))
        cpu["one_thread"] = round(n1 / (time.perf_counter() - s0), 1)
        ref.set_threads(threads)

    line = {
        "metric": "variant-selection decisions/sec on 1 MI355X; % of HBM roofline",
        "value": round(value, 1), "unit": "decisions/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"config {cfg} ({spec['name']}): {tb.num_tasks} tasks, {tb.V} variants, "
                               f"{tb.B} batch sizes, {per_step} queries per step"
                               + (f", table bent to {args.table}" if args.table != "config" else "")
                               + (", after a load report that makes every variant a possible answer" if args.degrade else "")
                               + f", rotating over {n_sets} batches and result arrays ({n_distinct} seeds)"
                               + (f", load report of {updates[0][2].variant_idx.size} rows before every step" if updates else "")
                               + (", closest-variant mode (two result arrays)" if args.closest else "")
                               + (", state-aware two-tier selection (variant and tier arrays)" if args.tiered else "")
                               + (", complete Case I: two tiers, then the closest variant (variant, tier and suggestion arrays)"
                                  if args.case1 else "")
                               + (f", two-tier selection with worker selection over {cluster.W} workers and "
                                  f"{cluster.I} instances (variant, tier and worker arrays)" if args.workers else "")
                               + (f", the whole of Case I: two tiers, the worker of every answer over {cluster.W} workers and "
                                  f"{cluster.I} instances, else the closest variant (variant, tier, worker and suggestion "
                                  "arrays)" if args.getvariant else ""),
                   "engine": args.engine, "launch": "hip graph replay" if args.graph else
                   (f"{args.streams} streams, a handle each" if args.streams > 1 else "stream"),
                   "timed_region": "library instrumentation off; kernel durations from a second pass of the same steps; "
                                   f"{args.preheat_ms:g} ms of the same steps before the warm-up steps"},
        "roofline": roofline,
        "whole_step_frac_of_hbm_roofline": round(whole_frac, 5),
        "kernels_ms_per_step": {k: round(v["total_ms"] / args.steps, 5) for k, v in active.items()},
        "cpu_baseline": cpu,
        "parity_sample_mismatches": mismatches,
        "index": {k: v for k, v in sel.info().items() if k.startswith("index") or k.startswith("lookup")},
    }
    print(json.dumps(line))
    sel.destroy()
    return 0 if not mismatches else 1


if __name__ == "__main__":
    sys.exit(main())
