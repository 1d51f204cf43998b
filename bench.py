#!/usr/bin/env python3
"""Benchmark of the sampling + feature-loading hot path on one MI355X.

A step = one minibatch: 3-layer LABOR-0 sampling (count, scan, fill, hash-unique, relabel per layer)
followed by the gather of the input-layer feature rows, on the papers100M-shaped synthetic graph
(111M vertices, ~3.2B directed edges, fp16 features of dim 128, batch 16384).  Graph, features and
seeds are resident in HBM before the timed region.  Prints ONE JSON line on stdout; progress goes to
stderr.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME] [--scale-down S] [--kappa KAPPA]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # B/s, MI355X HBM3E
# plain-ALU ceiling for 32-bit integer work: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second
ALU_PEAK_INT32 = 256 * 4 * 16 * 2.4e9


def log(msg):
    print("[bench %7.1fs] %s" % (time.time() - T0, msg), file=sys.stderr, flush=True)


T0 = time.time()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="papers100M", choices=["tiny", "products", "reddit", "papers100M", "mag240M"])
    ap.add_argument("--scale-down", type=int, default=1, help="shrink the graph (development only; the result is then "
                    "labelled with the reduced workload)")
    ap.add_argument("--kappa", type=int, default=1)
    ap.add_argument("--sampler", default=None, choices=[None, "labor0", "ns", "rw"],
                    help="rw: random walks with the paper's parameters (length 3, 100 walks, restart probability 0.5)")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--mode", default="step", choices=["step", "batch-sweep", "kappa-cache", "host-cache", "mean-agg", "owner-bucket"],
                    help="step: the benchmark contract (default).  batch-sweep: |S^l| against batch size on nested seed prefixes "
                         "(products-shaped).  kappa-cache: LRU miss rate against kappa over consecutive dependent batches "
                         "(papers100M-shaped, 4M-row cache).  host-cache: pinned-host feature table behind a 32M-row cache "
                         "(mag240M-shaped), host-link bytes saved by kappa.")
    ap.add_argument("--iters", type=int, default=None, help="iterations per kappa for the cache modes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="step mode: skip the configuration's other workloads (kappa 16 / 256, NS, the two-stream pipeline) that the "
                         "default line times after the headline; for profiler runs, whose per-kernel sums should hold one workload")
    ap.add_argument("--plain-graph", action="store_true",
                    help="step mode: register the graph without COOP_SYMMETRIC (every list is then scanned)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB copies with the library's copy kernel (coop::k_copy_i32): the known-size "
                         "reference that rocprofv3 --pmc byte counters are scaled by")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the oracle timing leg")
    ap.add_argument("--tune", action="append", default=[], metavar="KNOB=VALUE",
                    help="coop_tune knob by number (see include/coop.h), e.g. --tune 2=16 for sixteen lists per wave; results never "
                         "depend on the knobs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one MI355X plays the single processor that owns the whole "
              "cooperative batch); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    import paper_2310_12403_amd as P

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    for kv in args.tune:
        knob, value = kv.split("=")
        P.coop_tune(int(knob), int(value))
    if args.mode != "step":
        return REPORTS[args.mode](args, torch, synth, P)
    dev = torch.device("cuda:0")
    cfg = dict(synth.CONFIGS[args.config])
    sampler_name = args.sampler or cfg["sampler"]
    sampler = {"labor0": P.COOP_LABOR0, "ns": P.COOP_NS, "rw": P.COOP_RW}[sampler_name]
    batch = args.batch or cfg["batch"]
    fanouts = cfg["fanouts"]
    dtype = torch.float16 if cfg["dtype"] == "f16" else torch.float32
    esize = 2 if cfg["dtype"] == "f16" else 4
    dim = cfg["dim"]

    # ---- inputs, resident in HBM --------------------------------------------------------------------------------
    log("building %s graph (scale_down=%d)" % (args.config, args.scale_down))
    indptr, indices = synth.make_graph(args.config, device=dev, scale_down=args.scale_down, log=log)
    torch.cuda.synchronize()
    n = indptr.numel() - 1
    nnz = indices.numel()
    log("graph: %d vertices, %d directed edges, max degree %d" % (n, nnz, int((indptr[1:] - indptr[:-1]).max())))
    feat = synth.features(n, dim, dtype, seed=0, device=dev)
    torch.cuda.synchronize()
    log("features: [%d, %d] %s = %.1f GB" % (n, dim, cfg["dtype"], n * dim * esize / 1e9))
    get_seeds = synth.seed_batches(n, batch, seed=0, device=dev)
    # (the synthetic graphs are undirected, stored both ways with sorted lists, like the bidirected benchmark graphs of the paper)
    symmetric = not args.plain_graph
    torch.cuda.synchronize()
    t_load = time.perf_counter()
    graph = P.coop_graph_load(indptr, indices, P.COOP_VALIDATE | (P.COOP_SYMMETRIC if symmetric else 0))
    load_ms = (time.perf_counter() - t_load) * 1e3
    arena = P.Arena(4 << 30)
    deg = indptr[1:] - indptr[:-1]

    def sample(i):
        if sampler == P.COOP_RW:
            return P.coop_sample_rw(graph, get_seeds(i), fanouts, *RW_PARAMS, it=i, seed=0, arena=arena)
        return P.coop_sample(graph, get_seeds(i), fanouts, sampler, it=i, kappa=args.kappa, seed=0, arena=arena)

    def step(i, out):
        arena.reset()
        blocks = sample(i)
        P.coop_gather(feat, blocks[-1].src_ids, out=out)        # writes the first n_src rows of the preallocated buffer
        return blocks

    # output buffer sized once from a dry run (allocation stays outside the timed region)
    arena.reset()
    probe = sample(0)
    out = torch.empty((int(probe[-1].n_src * 1.25) + 1024, dim), dtype=dtype, device=dev)
    log("probe: " + ", ".join("|S^%d|=%d |E^%d|=%d" % (l + 1, b.n_src, l, b.n_edges) for l, b in enumerate(probe)))

    if args.copy_calibration:
        a = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            P.coop_copy_ids(a, out=b)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b

    for i in range(args.warmup):
        step(i, out)
    P.coop_gather_status()
    torch.cuda.synchronize()

    # ---- per-kernel pass (all kernels timed with HIP events; not the timed region) -------------------------------
    P.profile_reset()
    P.profile_filter(None)
    P.profile_enable(True)
    for i in range(min(args.steps, 10)):
        step(args.warmup + i, out)
    torch.cuda.synchronize()
    P.profile_enable(False)
    per_kernel = P.profile_read_all()
    n_prof = min(args.steps, 10)
    breakdown = {k: round(v[0] / n_prof, 4) for k, v in sorted(per_kernel.items(), key=lambda kv: -kv[1][0])}
    dominant = next(iter(breakdown))
    log("per-kernel ms/step: " + json.dumps(breakdown))

    # ---- timed region: exactly K steps; only the dominant kernel carries events ------------------------------------
    P.profile_reset()
    P.profile_filter(dominant)
    P.profile_enable(True)
    stats = dict(edges=0, uniq=0, n_in=0, D=[0] * len(fanouts), n_l=[0] * len(fanouts), m_l=[0] * len(fanouts),
                 n_src=[0] * len(fanouts))
    kept = []
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        blocks = step(args.warmup + i, out)
        kept.append([(b.n_dst, b.n_edges, b.n_src) for b in blocks])
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_start
    P.profile_enable(False)
    P.coop_gather_status()
    dom_ms, dom_launches = P.profile_read_all()[dominant]
    P.profile_filter(None)

    for sizes in kept:
        for l, (nd, m, ns) in enumerate(sizes):
            stats["n_l"][l] += nd
            stats["m_l"][l] += m
            stats["n_src"][l] += ns
        stats["edges"] += sum(m for _, m, _ in sizes)
        stats["uniq"] += sum(ns for _, _, ns in sizes)
        stats["n_in"] += sizes[-1][2]
    K = args.steps
    ms_per_step = t_total / K * 1e3

    # neighbours examined per layer (D_l = sum of degrees over S^l), measured on the last step's blocks
    D_last = [int(deg[b.dst_ids.long()].sum()) for b in blocks]
    n_last = [b.n_dst for b in blocks]
    m_last = [b.n_edges for b in blocks]
    nL_last = blocks[-1].n_src
    row_bytes = dim * esize

    # ---- algorithmic bytes (what the method must move) -------------------------------------------------------------
    def rw_walk_bytes(nl):   # per destination: id + list record, 4 B per step, a 16 B list record per step that does not restart
        o, a, p = RW_PARAMS
        return nl * (20 + 4 * o * a + 16 * a * (o - 1) * (1 - p))

    def sample_bytes(nl, Dl, ml, nsrc):
        count_fill = 16 * nl + 4 * nl + 4 * Dl + 8 * (nl + 1) + 4 * ml + 8 * ml
        if sampler == P.COOP_RW:
            count_fill = rw_walk_bytes(nl) + 8 * (nl + 1) + 12 * ml
        unique = 4 * ml + 8 * (nl + ml) + 8 * ml + 4 * (nsrc - nl) + 4 * ml
        return count_fill + unique

    alg_sample = sum(sample_bytes(n_last[l], D_last[l], m_last[l], blocks[l].n_src) for l in range(len(fanouts)))
    alg_gather = 2 * nL_last * row_bytes + 4 * nL_last
    step_frac = (alg_sample + alg_gather) / (ms_per_step * 1e-3) / HBM_PEAK

    avg_dom_ms = dom_ms / max(dom_launches, 1)
    if dominant == "gather":
        alg_dom = (2 * row_bytes + 4) * (stats["n_in"] / K)           # per launch: one gather per step
        roofline = dict(bound="hbm", kernel=dominant, achieved=alg_dom / (avg_dom_ms * 1e-3) / 1e9, peak=HBM_PEAK / 1e9,
                        unit="GB/s")
    elif dominant == "labor_scan":
        # The scan reads every neighbour list once per minibatch: pass l covers the destinations new at layer l and
        # evaluates layers l..L-1 together.  Per launch: a 16-byte list record and (threshold + count) per covered layer
        # for each new destination, 4 bytes per neighbour examined.
        # On a graph registered as symmetric, with independent variates and fanouts up to 64, a pass over 65536 lists or
        # more leaves the lists longer than 8192 to the kernels that work from the neighbours' side: the scan never
        # reads them, and they are not counted here.
        Lf = len(fanouts)
        per_step = 0
        per_step_every_list = 0
        covered = 0                    # the library's pass rule: a pass over fewer than 32768 lists covers its own layer only
        # (and only on a graph whose lists above 8192 hold an eighth of the edges or more)
        other_side = (symmetric and sampler == P.COOP_LABOR0 and args.kappa == 1 and max(fanouts) <= 64
                      and int(deg[deg > 8192].sum()) * 8 >= nnz)
        for l in range(Lf):
            n_new = n_last[l] - covered
            d_new = deg[blocks[l].dst_ids[covered:].long()]
            fused = n_new >= 32768 or l == Lf - 1
            nf = Lf - l if fused else 1
            per_step_every_list += 16 * n_new + 8 * nf * n_new + 4 * int(d_new.sum())
            if other_side and n_new >= 65536:
                d_new = d_new[d_new <= 8192]
            per_step += 16 * n_new + 8 * nf * n_new + 4 * int(d_new.sum())
            if fused:
                covered = n_last[l]
        alg_dom = per_step / Lf
        roofline = dict(bound="hbm", kernel=dominant, achieved=alg_dom / (avg_dom_ms * 1e-3) / 1e9, peak=HBM_PEAK / 1e9,
                        unit="GB/s")
        # Beside it: the count stage as a whole (the scan and, on a symmetric graph, the two kernels that stand in for the
        # scan of the longest lists) against the bytes of a scan that reads every list once (4 bytes per neighbour of
        # every destination of the last layer).  Times from the per-kernel pass (HIP events around every launch).
        stage_ms = sum(breakdown.get(k, 0.0) for k in ("labor_scan", "enum_list", "enum_walk"))
        count_stage = dict(kernels=[k for k in ("labor_scan", "enum_list", "enum_walk") if k in breakdown], ms_per_step=round(stage_ms, 4),
                           bytes_every_list_once=per_step_every_list,
                           effective_GBps=round(per_step_every_list / (stage_ms * 1e-3) / 1e9, 1),
                           effective_frac=round(per_step_every_list / (stage_ms * 1e-3) / HBM_PEAK, 4))
    elif dominant == "rw_walk":
        alg_dom = sum(rw_walk_bytes(n_last[l]) + 4 * n_last[l] + 8 * m_last[l] for l in range(len(fanouts))) / len(fanouts)
        roofline = dict(bound="hbm", kernel=dominant, achieved=alg_dom / (avg_dom_ms * 1e-3) / 1e9, peak=HBM_PEAK / 1e9,
                        unit="GB/s")
    elif dominant in ("labor_fill", "ns_fill"):
        per_step = sum(24 * n_last[l] + (4 * D_last[l] if dominant == "ns_fill" else 0) + 12 * m_last[l] for l in range(len(fanouts)))
        alg_dom = per_step / len(fanouts)
        roofline = dict(bound="hbm", kernel=dominant, achieved=alg_dom / (avg_dom_ms * 1e-3) / 1e9, peak=HBM_PEAK / 1e9,
                        unit="GB/s")
    else:
        per_step = sum(4 * m_last[l] + 8 * (n_last[l] + m_last[l]) for l in range(len(fanouts)))
        alg_dom = per_step / len(fanouts)
        roofline = dict(bound="hbm", kernel=dominant, achieved=alg_dom / (avg_dom_ms * 1e-3) / 1e9, peak=HBM_PEAK / 1e9,
                        unit="GB/s")
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    roofline["avg_launch_ms"] = avg_dom_ms
    roofline["launches"] = dom_launches
    roofline["algorithmic_bytes_per_launch"] = alg_dom
    roofline["traffic"] = _stored_traffic(dominant + ("_plain_graph" if dominant == "labor_scan" and not symmetric else ""), args)
    step_traffic = _stored_traffic("step_all_kernels", args) if (symmetric and sampler == P.COOP_LABOR0 and args.kappa == 1) else None
    roofline["achieved"] = round(roofline["achieved"], 2)
    roofline["frac"] = round(roofline["frac"], 4)

    workload = "%s-shaped Chung-Lu graph (%d vertices, %d directed edges), %d-layer %s fanout %s, batch %d, %s dim %d, kappa %d" % (
        args.config, n, nnz, len(fanouts), sampler_name.upper(), "/".join(map(str, fanouts)), batch, cfg["dtype"], dim, args.kappa)
    if args.scale_down != 1:
        workload += " [REDUCED: scale_down=%d, development run]" % args.scale_down
    result = {
        "metric": "sampled edges/s + feature-gather GB/s (% HBM peak), 3-layer " + {"labor0": "LABOR-0", "ns": "NS", "rw": "RW"}[sampler_name],
        "value": round(stats["edges"] / t_total, 1),
        "unit": "sampled edges/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 variates / int32 ids / %s rows (copied bit-exactly)" % cfg["dtype"],
        "data": "synthetic",
        "config": {"workload": workload, "sampler": sampler_name, "fanouts": list(fanouts), "batch": batch,
                   "kappa": args.kappa, "feature_dim": dim, "feature_dtype": cfg["dtype"]},
        "unique_vertices_per_s": round(stats["uniq"] / t_total, 1),
        "input_vertices_per_step": round(stats["n_in"] / K, 1),
        "sampled_edges_per_step": round(stats["edges"] / K, 1),
        "sizes_last_step": {"n_dst": n_last, "neighbours_examined": D_last, "n_edges": m_last,
                            "n_src": [b.n_src for b in blocks]},
        "per_kernel_ms_per_step": breakdown,
        "gather_GBps": round((2 * row_bytes) * (stats["n_in"] / K) / (breakdown.get("gather", float("nan")) * 1e-3) / 1e9, 1),
        # two views of the whole step.  "layerwise" = the algorithmic bytes of a sampler that works layer by layer (every
        # list of S^l charged at every layer l), divided by the step time: an EFFECTIVE rate,
        # which the fused scan and the lists served from the neighbours' side undercut.  "measured" = HBM bytes actually
        # moved by all kernels of a step (rocprofv3 FETCH_SIZE / WRITE_SIZE summary under profiles/), divided by the same
        # step time: the achieved bandwidth.
        "step_layerwise_bytes": alg_sample + alg_gather,
        "step_hbm_frac_effective_layerwise_bytes": round(step_frac, 4),
        "step_traffic_bytes": step_traffic,
        "step_hbm_frac_measured": None if step_traffic is None else round(step_traffic / (ms_per_step * 1e-3) / HBM_PEAK, 4),
        "roofline": roofline,
    }
    if dominant == "labor_scan":
        result["count_stage"] = count_stage
    if symmetric and sampler == P.COOP_LABOR0:
        result["reverse_index"] = {"bytes": 4 * nnz, "build_ms": round(load_ms, 1),
                                   "note": "COOP_SYMMETRIC registration: one uint32 per edge, built once per graph, outside the timed region"}

    # ---- CPU baseline: the oracle as it stands, on the host cores of this machine ----------------------------------------
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, indptr, indices, feat, get_seeds, fanouts, sampler, blocks, K, P)

    # ---- the configuration's other workloads, timed the same way (K steps between two synchronisations); after the oracle's
    # comparison, which reads the last timed step's blocks in the arena that these steps reuse --------------------------------
    if args.config == "papers100M" and sampler == P.COOP_LABOR0 and args.kappa == 1 and not args.plain_graph and not args.headline_only:
        def timed(sample_fn):
            arena.reset()
            rows = torch.empty((int(sample_fn(0)[-1].n_src * 1.25) + 1024, dim), dtype=dtype, device=dev)   # sized from a dry run

            def one(i):
                arena.reset()
                P.coop_gather(feat, sample_fn(i)[-1].src_ids, out=rows)

            for i in range(3):
                one(i)
            torch.cuda.synchronize()
            t = time.perf_counter()
            for i in range(K):
                one(args.warmup + i)
            torch.cuda.synchronize()
            return round((time.perf_counter() - t) / K * 1e3, 4)

        def dependent(kappa):
            return lambda i: P.coop_sample(graph, get_seeds(i), fanouts, P.COOP_LABOR0, it=i * kappa + kappa // 3 + 1, kappa=kappa, seed=0,
                                           arena=arena)

        def ns_step(i):
            return P.coop_sample(graph, get_seeds(i), fanouts, P.COOP_NS, it=i, kappa=1, seed=0, arena=arena)

        # the same kappa = 1 steps as a two-deep pipeline: consecutive steps alternate between two streams (each with an
        # arena and an output buffer of its own, default priority), so that the gather of one batch, which is bound by
        # bandwidth, runs beside the sampling of the next, which is not.  Reported beside the headline, which stays the
        # one-stream figure (the dominant kernel's duration is timed there, by itself).
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        arenas = [arena, P.Arena(4 << 30)]
        outs = [out, torch.empty_like(out)]

        def piped(i):
            st = streams[i & 1]
            arenas[i & 1].reset()
            b = P.coop_sample(graph, get_seeds(i), fanouts, P.COOP_LABOR0, it=i, kappa=1, seed=0, arena=arenas[i & 1], stream=st)
            P.coop_gather(feat, b[-1].src_ids, out=outs[i & 1], stream=st)

        torch.cuda.synchronize()
        for i in range(4):
            piped(i)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(K):
            piped(args.warmup + i)
        torch.cuda.synchronize()
        result["two_stream_pipeline_ms_per_step"] = round((time.perf_counter() - t) / K * 1e3, 4)
        del arenas, outs
        result["kappa16_ms_per_step"] = timed(dependent(16))     # dependent variates, c = 6/16 (every step inside a group)
        result["kappa256_ms_per_step"] = timed(dependent(256))   # c = 86/256
        result["ns_ms_per_step"] = timed(ns_step)                # NS 10/10/10 on the same batches
        P.coop_gather_status()
        log("kappa 16: %.3f ms, kappa 256: %.3f ms, NS: %.3f ms per step" % (result["kappa16_ms_per_step"], result["kappa256_ms_per_step"],
                                                                           result["ns_ms_per_step"]))

    print(json.dumps(result), flush=True)


def report_batch_sweep(args, torch, synth, P):
    """|S^l| against batch size (Thm 3.1 / 3.2 and the paper's first experiment): products-shaped graph, 3-layer
    LABOR-0, batches that are nested prefixes of one seed permutation, several permutations."""
    import numpy as np
    dev = torch.device("cuda:0")
    name = "products" if args.config == "papers100M" else args.config
    cfg = synth.CONFIGS[name]
    indptr, indices = synth.make_graph(name, device=dev, scale_down=args.scale_down, log=log)
    n = indptr.numel() - 1
    # (the synthetic graphs are undirected, stored both ways with sorted lists, like the bidirected benchmark graphs of the paper)
    graph = P.coop_graph_load(indptr, indices, P.COOP_VALIDATE | P.COOP_SYMMETRIC)
    arena = P.Arena(2 << 30)
    sizes = [1024, 4096, 16384, 65536]
    perms = 8
    acc = np.zeros((len(sizes), len(cfg["fanouts"])))
    ms = np.zeros(len(sizes))
    nested_ok = True
    warm = synth.permutation(n, 899, device=dev).to(torch.int32)
    for b in sizes:  # (untimed: the first launch of every kernel loads its code)
        arena.reset()
        P.coop_sample(graph, warm[:b].contiguous(), cfg["fanouts"], P.COOP_LABOR0, it=0, kappa=1, seed=0, arena=arena)
    for p in range(perms):
        perm = synth.permutation(n, 900 + p, device=dev).to(torch.int32)
        prev_sets = None
        for i, b in enumerate(sizes):
            arena.reset()
            torch.cuda.synchronize()
            t = time.perf_counter()
            blocks = P.coop_sample(graph, perm[:b].contiguous(), cfg["fanouts"], P.COOP_LABOR0, it=p, kappa=1, seed=p, arena=arena)
            torch.cuda.synchronize()
            ms[i] += (time.perf_counter() - t) * 1e3
            acc[i] += [blk.n_src for blk in blocks]
            if p == 0:      # exact nestedness: the smaller batch's S^l is a subset of the larger batch's
                sets = [blk.src_ids.clone() for blk in blocks]
                if prev_sets is not None:
                    for small, big in zip(prev_sets, sets):
                        nested_ok = nested_ok and bool(torch.isin(small, big).all())
                prev_sets = sets
    acc /= perms
    ms /= perms
    ratio = acc / np.array(sizes)[:, None]
    result = {"report": "batch-sweep", "workload": "%s-shaped Chung-Lu graph (%d vertices, %d directed edges), 3-layer LABOR-0 %s, kappa 1" % (
                  name, n, indices.numel(), "/".join(map(str, cfg["fanouts"]))),
              "batch_sizes": sizes, "mean_S_l": acc.round(1).tolist(), "S_l_per_seed": ratio.round(3).tolist(),
              "work_per_seed_nonincreasing": bool((np.diff(ratio, axis=0) < 0).all()),
              "increments_concave": bool((np.diff(acc, axis=0)[1:] <= 4 * np.diff(acc, axis=0)[:-1] * 1.02).all()),
              "nested_exactly": nested_ok, "ms_per_batch": ms.round(3).tolist(), "permutations": perms}
    print(json.dumps(result), flush=True)


def _cache_run(args, torch, synth, P, graph, n, get_seeds, fanouts, table, cache_rows, dim, dtype, kappas, iters, check_iters):
    from oracle import coopref as R
    out_rows = None
    res = {}
    for kappa in kappas:
        arena = P.Arena(6 << 30)
        cache = P.Cache(cache_rows, n, dim, dtype, max_ids=16 << 20)
        oracle = R.Cache(cache_rows, n) if check_iters else None
        misses, totals, t_sample, t_gather, agree = [], [], 0.0, 0.0, True
        for it in range(iters):
            arena.reset()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            blocks = P.coop_sample(graph, get_seeds(it), fanouts, P.COOP_LABOR0, it=it, kappa=kappa, seed=0, arena=arena)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            ids = blocks[-1].src_ids
            if out_rows is None or out_rows.shape[0] < ids.numel():
                out_rows = torch.empty((int(ids.numel() * 1.3), dim), dtype=dtype, device=ids.device)
            _, n_miss = cache.gather(table, ids, out=out_rows[:ids.numel()])
            torch.cuda.synchronize()     # the miss rows may still be streaming in when the call returns
            t2 = time.perf_counter()
            if it >= iters // 4:
                t_sample += t1 - t0
                t_gather += t2 - t1
            misses.append(n_miss)
            totals.append(ids.numel())
            if oracle is not None and (check_iters is None or it < check_iters):
                want, _ = oracle.access(ids.cpu().numpy())
                agree = agree and want == n_miss
        # per-kernel times of the cached gather alone, a few more iterations of the same run (HIP events around every launch)
        P.profile_reset()
        P.profile_filter(None)
        n_prof = min(8, iters)
        for it in range(iters, iters + n_prof):
            arena.reset()
            ids = P.coop_sample(graph, get_seeds(it), fanouts, P.COOP_LABOR0, it=it, kappa=kappa, seed=0, arena=arena)[-1].src_ids
            if out_rows.shape[0] < ids.numel():
                out_rows = torch.empty((int(ids.numel() * 1.3), dim), dtype=dtype, device=ids.device)
            torch.cuda.synchronize()
            P.profile_enable(True)
            cache.gather(table, ids, out=out_rows[:ids.numel()])
            torch.cuda.synchronize()
            P.profile_enable(False)
        kernels = {k: round(v[0] / n_prof, 4) for k, v in sorted(P.profile_read_all().items(), key=lambda kv: -kv[1][0])}
        tail = iters // 4
        res[str(kappa)] = {"cache_kernels_ms_per_call": kernels,
                           "miss_rate_all": round(sum(misses) / sum(totals), 4),
                           "miss_rate_steady": round(sum(misses[tail:]) / sum(totals[tail:]), 4),
                           "mean_input_vertices": round(sum(totals) / iters, 1),
                           "misses_per_iter_steady": round(sum(misses[tail:]) / (iters - tail), 1),
                           "ms_sample_steady": round(t_sample / (iters - tail) * 1e3, 3),
                           "ms_cache_gather_steady": round(t_gather / (iters - tail) * 1e3, 3),
                           ("oracle_lru_agrees_all_%d_iters" % iters if check_iters is None else "oracle_lru_agrees_first_%d_iters" % check_iters): agree}
        log("kappa %d: %s" % (kappa, json.dumps(res[str(kappa)])))
        cache.close()
        del cache, arena
    return res


def report_kappa_cache(args, torch, synth, P):
    """LRU miss rate against kappa (Sec. 4.2).  Default: papers100M-shaped graph, LABOR-0 10/10/10, batch 16384, consecutive
    dependent batches, 4M-row vertex cache in front of the HBM-resident feature table.  With --config reddit: the setting of
    the one miss rate that the paper quotes (reddit, one GPU, batch 1024, fanout 10, 3 layers, 60,000-row cache), on the
    reddit-shaped graph."""
    dev = torch.device("cuda:0")
    name = "reddit" if args.config == "reddit" else "papers100M"
    cfg = synth.CONFIGS[name]
    indptr, indices = synth.make_graph(name, device=dev, scale_down=args.scale_down, log=log)
    n = indptr.numel() - 1
    graph = P.coop_graph_load(indptr, indices, P.COOP_SYMMETRIC)
    dtype = torch.float16 if cfg["dtype"] == "f16" else torch.float32
    feat = synth.features(n, cfg["dim"], dtype, seed=0, device=dev)
    batch = args.batch or (1024 if name == "reddit" else cfg["batch"])
    fanouts = (10, 10, 10)
    get_seeds = synth.seed_batches(n, batch, seed=0, device=dev)
    iters = args.iters or 512
    cache_rows = (60000 if name == "reddit" else 4000000) // args.scale_down
    kappas = (1, 4, 16, 64, 256, 0) if name == "reddit" else (1, 16, 256)
    res = _cache_run(args, torch, synth, P, graph, n, get_seeds, fanouts, feat, cache_rows, cfg["dim"], dtype,
                     kappas, iters, check_iters=None)   # the oracle's LRU follows every iteration
    print(json.dumps({"report": "kappa-cache", "workload": "%s-shaped graph (%d vertices, %d directed edges), 3-layer LABOR-0 "
                      "10/10/10, batch %d, %d consecutive iterations per kappa (kappa 0 = infinity), %d-row LRU cache, %s x %d rows in HBM; "
                      "'steady' skips the first quarter of the iterations" % (name, n, indices.numel(), batch, iters, cache_rows,
                                                                             cfg["dtype"], cfg["dim"]),
                      "by_kappa": res}), flush=True)


def report_host_cache(args, torch, synth, P):
    """Pinned-host feature table behind an on-GPU cache: mag240M-shaped graph, LABOR-0 10/10/10, batch 32768, kappa 1 and 64.
    The full fp16 x 768 table (375 GB) does not fit this machine's host memory: a shorter pinned table is aliased (vertex v
    reads row v mod R) while the cache is keyed by v, so miss counts and bytes per miss are those of the full table."""
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS["mag240M"]
    indptr, indices = synth.make_graph("mag240M", device=dev, scale_down=args.scale_down, log=log)
    n = indptr.numel() - 1
    graph = P.coop_graph_load(indptr, indices, P.COOP_SYMMETRIC)
    R_rows = (32 << 20) // args.scale_down
    log("pinned host table: %d rows x %d fp16 = %.1f GB" % (R_rows, cfg["dim"], R_rows * cfg["dim"] * 2 / 1e9))
    table = torch.empty((R_rows, cfg["dim"]), dtype=torch.float16, pin_memory=True)
    chunk = 1 << 19
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    for lo in range(0, R_rows, chunk):   # N(0,1) rows drawn on the GPU, copied down into the pinned table
        rows = min(chunk, R_rows - lo)
        table[lo:lo + rows].copy_(torch.randn((rows, cfg["dim"]), generator=g, device=dev).to(torch.float16))
    get_seeds = synth.seed_batches(n, cfg["batch"], seed=0, device=dev)
    iters = args.iters or 48
    cache_rows = 32000000 // args.scale_down
    res = _cache_run(args, torch, synth, P, graph, n, get_seeds, cfg["fanouts"], table, cache_rows, cfg["dim"], torch.float16,
                     (1, 64), iters, check_iters=4)
    row_bytes = cfg["dim"] * 2
    for k, v in res.items():
        v["host_link_GB_per_iter_steady"] = round(v["misses_per_iter_steady"] * row_bytes / 1e9, 4)
        v["host_link_GBps_steady"] = round(v["misses_per_iter_steady"] * row_bytes / (v["ms_cache_gather_steady"] * 1e-3) / 1e9, 2)
    saved = (res["1"]["misses_per_iter_steady"] - res["64"]["misses_per_iter_steady"]) * row_bytes / 1e9
    print(json.dumps({"report": "host-cache", "workload": "mag240M-shaped graph (%d vertices, %d directed edges), 3-layer LABOR-0 "
                      "10/10/10, batch %d, %d iterations per kappa, %d-row cache, fp16 x %d rows read from a %d-row pinned host table "
                      "(aliased)" % (n, indices.numel(), cfg["batch"], iters, cache_rows, cfg["dim"], R_rows),
                      "by_kappa": res, "host_link_GB_saved_per_iter_kappa64_vs_1": round(saved, 4)}), flush=True)


def report_mean_agg(args, torch, synth, P):
    """Neighbour mean over the last block fused with the feature load, against gather-then-nothing: papers100M-shaped."""
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS["papers100M"]
    indptr, indices = synth.make_graph("papers100M", device=dev, scale_down=args.scale_down, log=log)
    n = indptr.numel() - 1
    graph = P.coop_graph_load(indptr, indices, P.COOP_SYMMETRIC)
    feat = synth.features(n, cfg["dim"], torch.float16, seed=0, device=dev)
    get_seeds = synth.seed_batches(n, cfg["batch"], seed=0, device=dev)
    arena = P.Arena(4 << 30)
    blocks = P.coop_sample(graph, get_seeds(0), cfg["fanouts"], P.COOP_LABOR0, it=0, kappa=1, seed=0, arena=arena)
    blk = blocks[-1]
    out_mean = torch.empty((blk.n_dst, cfg["dim"]), dtype=torch.float16, device=dev)
    out_rows = torch.empty((blk.n_src, cfg["dim"]), dtype=torch.float16, device=dev)
    row_bytes = cfg["dim"] * 2
    res = {}
    for name, fn, nbytes in (("gather_mean", lambda: P.coop_gather_mean(feat, blk.indptr, blk.col_global, out=out_mean),
                              blk.n_edges * (row_bytes + 4) + blk.n_dst * (row_bytes + 8)),
                             ("gather", lambda: P.coop_gather(feat, blk.src_ids, out=out_rows), blk.n_src * (2 * row_bytes + 4))):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t) / 20 * 1e3
        res[name] = {"ms": round(ms, 4), "algorithmic_GB": round(nbytes / 1e9, 4), "GBps": round(nbytes / ms / 1e6, 1),
                     "hbm_frac": round(nbytes / (ms * 1e-3) / HBM_PEAK, 4)}
    P.coop_gather_status()
    if not args.no_cpu_baseline:
        from oracle import coopref as R
        import numpy as np
        k = 2000   # the first destinations of the block against the oracle's fp64 mean
        ip = blk.indptr[:k + 1].cpu().numpy()
        want = R.gather_mean(feat.cpu().numpy(), ip, blk.col_global[:int(ip[-1])].cpu().numpy())
        got = out_mean[:k].float().cpu().numpy().astype(np.float64)
        scale = np.maximum(np.abs(want).max(axis=1, keepdims=True), 1e-30)
        res["max_rel_err_vs_oracle_first_%d_rows" % k] = float(np.max(np.abs(got - want) / scale))
    print(json.dumps({"report": "mean-agg", "workload": "papers100M-shaped graph, last block of a 3-layer LABOR-0 batch of %d: "
                      "%d destinations, %d edges, %d source rows, fp16 x %d" % (cfg["batch"], blk.n_dst, blk.n_edges, blk.n_src, cfg["dim"]),
                      "kernels": res}), flush=True)


def report_owner_bucket(args, torch, synth, P):
    """The local half of the id redistribution (Sec. 3.1): the input frontier S^3 of a papers100M-shaped batch grouped by
    the owning PE of an 8-way vertex partition (contiguous ranges, and the random partition)."""
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS["papers100M"]
    indptr, indices = synth.make_graph("papers100M", device=dev, scale_down=args.scale_down, log=log)
    n = indptr.numel() - 1
    graph = P.coop_graph_load(indptr, indices, P.COOP_SYMMETRIC)
    get_seeds = synth.seed_batches(n, cfg["batch"], seed=0, device=dev)
    arena = P.Arena(4 << 30)
    blocks = P.coop_sample(graph, get_seeds(0), cfg["fanouts"], P.COOP_LABOR0, it=0, kappa=1, seed=0, arena=arena)
    ids = blocks[-1].src_ids.clone()
    n_ids, n_parts = ids.numel(), 8
    work = torch.empty(1 << 22, dtype=torch.uint8, device=dev)
    res = {}
    for name, scheme in (("ranges", P.COOP_OWNER_RANGE), ("hashed", P.COOP_OWNER_HASH)):
        for _ in range(3):
            out = P.coop_bucket_by_owner(ids, n, n_parts, scheme, seed=1, workspace=work)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(20):
            out = P.coop_bucket_by_owner(ids, n, n_parts, scheme, seed=1, workspace=work)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t) / 20 * 1e3
        nbytes = 16 * n_ids   # the ids read twice (count, place), the grouped ids and their origins written
        res[name] = {"ms": round(ms, 4), "ids_per_s": round(n_ids / ms * 1e3, 1), "algorithmic_GB": round(nbytes / 1e9, 4),
                     "GBps": round(nbytes / ms / 1e6, 1), "group_sizes": [int(x) for x in torch.diff(out[2]).cpu()]}
        if not args.no_cpu_baseline:
            from oracle import coopref as R
            import numpy as np
            want = R.bucket_by_owner(ids.cpu().numpy(), n, n_parts, scheme, seed=1)
            res[name]["matches_oracle"] = all(np.array_equal(a.cpu().numpy(), w) for a, w in zip(out, want))
    P.coop_gather_status()
    print(json.dumps({"report": "owner-bucket", "workload": "papers100M-shaped graph, S^3 of a 3-layer LABOR-0 batch of %d: %d ids, "
                      "%d owners" % (cfg["batch"], n_ids, n_parts), "partitions": res}), flush=True)


REPORTS = {"owner-bucket": report_owner_bucket, "mean-agg": report_mean_agg, "batch-sweep": report_batch_sweep, "kappa-cache": report_kappa_cache, "host-cache": report_host_cache}


def _stored_traffic(kernel, args):
    """HBM bytes per launch measured offline with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), if a summary for this
    kernel and workload has been recorded under profiles/; else None."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if args.scale_down != 1 or not os.path.exists(path):
        return None
    try:
        table = json.load(open(path))
        return table.get(args.config, {}).get(kernel)
    except Exception:
        return None


RW_PARAMS = (3, 100, 0.5)   # walk length, walks per destination, restart probability (the paper's experimental setup)


def cpu_baseline(args, indptr, indices, feat, get_seeds, fanouts, sampler, last_blocks, K, P):
    """Times oracle sampling + gather on a bounded sample of the same workload: whole batches, the same seeds and
    iteration numbers as the timed region's last steps, until the time budget is used.  Also confirms that the GPU
    blocks of the last timed step equal the oracle's (all arrays)."""
    import numpy as np
    from oracle import coopref as R

    log("cpu baseline: copying CSR and features to the host")
    ip_h = indptr.cpu().numpy()
    ix_h = indices.cpu().numpy()
    feat_h = feat.cpu().numpy()
    log("cpu baseline: running the oracle")
    edges, spent, batches, parity = 0, 0.0, 0, None
    i = args.warmup + K - 1
    while spent < args.cpu_seconds and batches < 8:
        seeds_h = get_seeds(i).cpu().numpy()
        t = time.perf_counter()
        blocks = R.sample(ip_h, ix_h, seeds_h, fanouts, sampler, it=i, kappa=args.kappa, seed=0, rw=RW_PARAMS)
        rows = R.gather(feat_h, blocks[-1]["src_ids"])
        spent += time.perf_counter() - t
        edges += sum(len(b["col_global"]) for b in blocks)
        if batches == 0:
            parity = all(np.array_equal(getattr(g, name).cpu().numpy(), w[name])
                         for g, w in zip(last_blocks, blocks)
                         for name in ("dst_ids", "indptr", "col_global", "eid", "col_local", "src_ids"))
            import torch
            got = P.coop_gather(feat, last_blocks[-1].src_ids)
            parity = parity and got.cpu().numpy().tobytes() == rows.tobytes()
            log("cpu baseline: GPU blocks of the last timed step equal the oracle's: %s" % parity)
        batches += 1
        i -= 1
        del rows, blocks
    single = {"value": round(edges / spent, 1), "unit": "sampled edges/s", "cores": 1, "kind": "oracle",
              "sample": "%d whole batches of the same workload (sampling + gather), %.1f s of single-thread CPU time" % (batches, spent),
              "matches_gpu_last_step": parity}
    # The same oracle on all host cores of this machine's share: one whole batch per thread, different batches side by side
    # (the oracle's C call releases the interpreter lock; the oracle itself stays the plain single-threaded code).
    from concurrent.futures import ThreadPoolExecutor
    cores = max(1, min(16, os.cpu_count() or 1))

    if args.kappa not in (0, 1):   # (with dependent variates one batch takes the oracle minutes: the single-thread figure stands alone)
        return single
    seeds_all = [get_seeds(args.warmup + K + j).cpu().numpy() for j in range(cores)]

    def one(j):
        blocks = R.sample(ip_h, ix_h, seeds_all[j], fanouts, sampler, it=args.warmup + K + j, kappa=args.kappa, seed=0, rw=RW_PARAMS)
        R.gather(feat_h, blocks[-1]["src_ids"])
        return sum(len(b["col_global"]) for b in blocks)

    t = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as pool:
        total = sum(pool.map(one, range(cores)))
    wall = time.perf_counter() - t
    single["all_cores"] = {"value": round(total / wall, 1), "unit": "sampled edges/s", "cores": cores, "kind": "oracle",
                           "sample": "%d whole batches, one per thread, side by side: %.1f s wall" % (cores, wall)}
    log("cpu baseline: %d threads, %.1f s wall, %.3g sampled edges/s" % (cores, wall, total / wall))
    return single


if __name__ == "__main__":
    main()
