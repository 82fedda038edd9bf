#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: sample -> reindex -> gather per batch.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload citation] [--streams S]

A step is one batch through sampling (all hops, dedup, relabel) and the gather of the feature rows
of every distinct sampled node.  In the timed region the batches go through qv_sample_many /
qv_gather_many, --batches-per-call independent batches per call (the paper's multiplexing of
several pipelines on one processor, Section 4.3), on --streams contexts.  p50 batch latency comes
from a separate pass with one batch per call.  All inputs (graph, features, seed batches) are
synthetic, seeded and resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, published
# Measured HBM bytes of k_gather over its algorithmic bytes (rocprofv3 FETCH_SIZE + WRITE_SIZE, each
# scaled by a 1 GiB plain copy kernel in the same run), keyed by workload, scale and id lists per
# k_gather launch; see GATHER_TRAFFIC_PROFILE.  Only quoted for configurations that were profiled.
GATHER_LISTS_PER_LAUNCH = 64
GATHER_TRAFFIC_RATIO = {("citation", 1.0, 64): 0.968, ("dense_social", 1.0, 64): 1.021, ("co_purchase", 1.0, 64): 1.156}
GATHER_TRAFFIC_PROFILE = ("profiles/citation_call_of_256_batches_kernels_and_counters.md and "
                          "profiles/other_workloads_kernel_durations_and_gather_traffic.md (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 "
                          "of k_gather over its algorithmic bytes, same workload and lists per launch)")


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def algorithmic_bytes(n_frontier_entries, n_edges, n_unique, n_rows, row_bytes, rowptr_bytes, tiered):
    """Bytes the method must move for one batch.  Per unit: a frontier entry costs its id, two row
    pointers and an 8-byte offset; a sampled edge 4 + 4 bytes in sampling and 4 + 8 + 8 in the
    reindex; a new node 4; a gathered row its id (and lookup entry when tiered), read and written."""
    sample = n_frontier_entries * (4 + 2 * rowptr_bytes + 8) + n_edges * (4 + 4)
    reindex = n_edges * (4 + 8 + 8) + n_unique * 4 + n_frontier_entries * 4
    gather = n_rows * (4 + (4 if tiered else 0) + 2 * row_bytes)
    return sample, reindex, gather


def psgs_curve(qv, qvgen, w, ctx, g, feat, Q, rowptr, col, tdtype):
    """One batch at a time: PSGS summed over the seeds (the paper's dispatch signal) against the
    measured latency of sample + gather on the GPU and of the oracle on one host core."""
    import numpy as np
    import torch
    import oracle
    assert Q is not None, "--psgs-curve needs the PSGS pass (do not pass --no-metrics)"
    sub_rows = min(w.n, 4_000_000)
    host_table = qvgen.features_host(w.seed, sub_rows, w.dim, w.feat_dtype)
    points = []
    for bs in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096):
        buf = qv.SampleBuffers(ctx, bs, w.fanouts, w.n)
        rows = feat.empty_rows(buf.caps[0], "cuda")
        plan = qv.ManyPlan(ctx, g, feat, [buf], [rows], w.fanouts)
        gpu_ms, cpu_ms, psgs, edges = [], [], [], []
        for rep in range(12):
            seeds = w.seeds(10_000 + rep, bs)
            d_seeds = torch.from_numpy(seeds).cuda()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(ctx.stream)
            plan.run([d_seeds], [w.rng_seed(rep)])
            e1.record(ctx.stream)
            ctx.sync()
            s = qv.qv_psgs_batch_sum(ctx, Q, d_seeds)
            ctx.sync()
            t1 = time.perf_counter()
            o = oracle.sample(rowptr, col, seeds, w.fanouts, w.rng_seed(rep))
            oracle.gather(host_table, o["n_id"] % sub_rows)
            t2 = time.perf_counter()
            if rep >= 2:                                   # the first runs size the scratch arena
                gpu_ms.append(e0.elapsed_time(e1)); cpu_ms.append((t2 - t1) * 1e3)
                psgs.append(s.item()); edges.append(int(o["edge_off"][-1]) + len(o["n_id"]))
        points.append({"batch": bs, "psgs_sum": round(float(np.mean(psgs)), 1),
                       "sampled_nodes_plus_edges": round(float(np.mean(edges)), 1),
                       "gpu_ms_avg": round(float(np.mean(gpu_ms)), 4), "gpu_ms_max": round(float(np.max(gpu_ms)), 4),
                       "cpu_oracle_ms_avg": round(float(np.mean(cpu_ms)), 4), "cpu_oracle_ms_max": round(float(np.max(cpu_ms)), 4)})
        log(str(points[-1]))
    print(json.dumps({"metric": "latency_vs_psgs", "workload": w.name, "cpu": "oracle, 1 core", "points": points}), flush=True)


def placement_ablation(qv, qvgen, w, ctx, g, table, P_pop, rowptr, col, tdtype):
    """Hot sets of the same size chosen by four rankings; HBM hit rate over Zipf-popular batches."""
    import numpy as np
    import torch
    assert w.hbm_budget is not None and P_pop is not None, "--placement-ablation needs the tiered workload and the FAP pass"
    deg_out = torch.from_numpy(np.diff(rowptr).astype(np.float32)).cuda()
    deg_in = torch.from_numpy(np.bincount(col, minlength=w.n).astype(np.float32)).cuda()
    rankings = {"fap_seed_popularity": P_pop, "fap_uniform_seeds": qv.qv_access_prob(ctx, g, w.fanouts),
                "in_degree": deg_in, "out_degree": deg_out}
    ctx.sync()
    n_hot = w.hbm_budget // w.row_bytes
    batches = []
    for b in range(16):
        seeds = torch.from_numpy(w.seeds(b)).cuda()
        out = qv.qv_sample(ctx, g, seeds, w.fanouts, w.rng_seed(b))
        ctx.sync()
        U = int(out.node_off[-1].item())
        batches.append(out.n_id[:U].clone())
    res = {}
    for name, score in rankings.items():
        rank = qv.qv_place_rank(ctx, score)
        ctx.sync()
        hot = torch.zeros(w.n, dtype=torch.bool, device="cuda")
        hot[rank[:n_hot].long()] = True
        hit = float(np.mean([hot[ids.long()].float().mean().item() for ids in batches]))
        feat = qv.Features(ctx, table, hbm_budget_bytes=w.hbm_budget, rank=rank)
        outs = [feat.empty_rows(ids.numel(), "cuda") for ids in batches[:8]]
        qv.qv_gather_many(ctx, feat, batches[:8], None, outs)
        ctx.sync()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(ctx.stream)
        qv.qv_gather_many(ctx, feat, batches[:8], None, outs)
        e1.record(ctx.stream)
        ctx.sync()
        rows = sum(ids.numel() for ids in batches[:8])
        res[name] = {"hbm_hit_rate": round(hit, 4), "gather_ms_8_batches": round(e0.elapsed_time(e1), 3),
                     "host_link_GBps": round((1 - hit) * rows * w.row_bytes / e0.elapsed_time(e1) / 1e6, 2)}
        # the same rows requested in address order (Section 5.3 sorts reads of slow tiers by address):
        # the cold tier holds its rows in ascending id order, so sorting the ids sorts the addresses
        sorted_ids = [ids.sort().values.contiguous() for ids in batches[:8]]
        qv.qv_gather_many(ctx, feat, sorted_ids, None, outs)
        ctx.sync()
        e0.record(ctx.stream)
        qv.qv_gather_many(ctx, feat, sorted_ids, None, outs)
        e1.record(ctx.stream)
        ctx.sync()
        res[name]["gather_ms_8_batches_address_sorted"] = round(e0.elapsed_time(e1), 3)
        log("%s: %s" % (name, res[name]))
        feat.close()
    print(json.dumps({"metric": "placement_ablation", "workload": w.name, "hot_rows": int(n_hot), "rankings": res}), flush=True)


def hardware_rates(qvgen):
    import torch
    import bench_probes
    out = {"metric": "hardware_rates", "unit": "1e9 operations/s", "rates": []}
    names = {0: "atomicMin u64 (result unused)", 1: "atomicMin u32 (result unused)", 2: "store 8 B", 3: "load 8 B",
             4: "atomicMin u64, workgroup scope", 5: "atomicMin u64, each XCD in its own eighth of the table",
             6: "atomicMin u64, workgroup scope, each XCD in its own eighth", 7: "load 8 B, each XCD in its own eighth"}
    xm = bench_probes.xcd_map(4096).cpu()
    out["workgroups_on_xcd_blockIdx_mod_8"] = int((xm == (torch.arange(4096, dtype=torch.int32) % 8)).sum().item())
    out["workgroups_checked"] = 4096
    for slots in (111_000_000, 1 << 23, 1 << 20):
        table = torch.full((slots,), -1, dtype=torch.int64, device="cuda")
        for n_ops in (1_000_000, 8_000_000):
            for mode in range(8):
                best = 1e9
                for rep in range(5):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    bench_probes.random_ops(mode, table, n_ops, salt=rep * 7919 + mode)
                    e1.record()
                    torch.cuda.synchronize()
                    best = min(best, e0.elapsed_time(e1))
                out["rates"].append({"op": names[mode], "table_slots": slots, "ops": n_ops, "us": round(best * 1e3, 1),
                                     "G_per_s": round(n_ops / best / 1e6, 1)})
                log(str(out["rates"][-1]))
        del table
    a = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
    b = torch.empty_like(a)
    best = 1e9
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        qvgen.copy_device(a, b)
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1))
    out["plain_copy_1GiB"] = {"ms": round(best, 4), "TB_per_s_read_plus_write": round(2 * a.numel() * 4 / best / 1e9, 3)}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="citation")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only)")
    ap.add_argument("--streams", type=int, default=1, help="batches in flight (one context per stream)")
    ap.add_argument("--extra-streams", type=int, default=16,
                    help="after the timed region, time the same region over 1, 2, 4, 8, 16 streams up to this many and "
                         "report ms per step for each (0 = skip; only when --streams is 1)")
    ap.add_argument("--batches-per-call", type=int, default=256,
                    help="independent batches per qv_sample_many / qv_gather_many call (1..256; halved while a call's "
                         "buffers would not fit the free device memory)")
    ap.add_argument("--latency-samples", type=int, default=200, help="single-batch calls timed for p50 / p99 (at least 200)")
    ap.add_argument("--table-budget-gib", type=float, default=-1.0,
                    help="dedup table budget per context in GiB for the table forms (0 = always hash; default: the library's 16)")
    ap.add_argument("--dedup", default="auto", choices=["auto", "table", "partitioned"],
                    help="dedup form of qv_sample (qv_ctx_set_dedup); results are identical")
    ap.add_argument("--partitions-log2", type=int, default=-1, help="partitions per batch of the partitioned form (-1: per call)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-metrics", action="store_true", help="skip the PSGS / FAP whole-graph passes")
    ap.add_argument("--psgs-curve", action="store_true",
                    help="instead of the benchmark: latency of one batch against the PSGS summed over its seeds "
                         "(Section 4.2.1), for batch sizes 1..4096, GPU path and CPU oracle side by side")
    ap.add_argument("--placement-ablation", action="store_true",
                    help="instead of the benchmark (tiered workload): HBM hit rate and gather time for hot sets "
                         "ranked by FAP under the seed popularity, FAP under uniform seeds, in-degree, out-degree; "
                         "each also with the ids sorted by address")
    ap.add_argument("--graph-in-host-memory", action="store_true",
                    help="keep rowptr / col in pinned host memory and sample through the host link (Section 4.3 (3))")
    ap.add_argument("--hardware-rates", action="store_true",
                    help="instead of the benchmark: rates of random device-scope atomics, stores and loads and of a "
                         "plain copy on this GPU (the yardsticks the dedup and gather kernels are priced against)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB copy kernel (copy_bytes) so that hardware byte counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported. "
              "Re-run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import qvgen
    import paper_2305_10863_amd as qv

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    qv.lib()
    torch.cuda.set_device(0)
    if args.hardware_rates:
        return hardware_rates(qvgen)
    w = qvgen.workload(args.workload, args.scale)
    batch = args.batch or w.batch
    K, W, S = args.steps, args.warmup, max(1, args.streams)

    # ---- inputs -----------------------------------------------------------------------------
    t0 = time.time()
    rowptr, col = w.graph()
    n_edges_graph = len(col)
    log("graph %s: %d nodes, %d edges generated in %.1fs" % (w.name, w.n, n_edges_graph, time.time() - t0))
    t0 = time.time()
    if args.graph_in_host_memory:      # zero-copy topology: the kernels read it over the host link
        d_rowptr, d_col = torch.from_numpy(rowptr).pin_memory(), torch.from_numpy(col).pin_memory()
    else:
        d_rowptr, d_col = torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda()
    tdtype = torch.float16 if w.feat_dtype == np.float16 else torch.float32
    table = qvgen.features_device(w.seed, w.n, w.dim, tdtype)
    torch.cuda.synchronize()
    log("graph uploaded, %.1f GB feature table filled in HBM in %.1fs" % (w.n * w.row_bytes / 1e9, time.time() - t0))

    if args.calibrate_copy:
        a = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            qvgen.copy_device(a, b)
        torch.cuda.synchronize()
        del a, b

    ctx0 = qv.Context(0)
    g = qv.Graph(ctx0, d_rowptr, d_col, validate=True)
    tiered = w.hbm_budget is not None and w.hbm_budget < w.n * w.row_bytes

    # ---- whole-graph metrics (deployment-time passes; not part of a step) ---------------------
    extra = {}
    Pdev = Qdev = None
    if not args.no_metrics:
        p0 = None
        if w.seed_mode == 1:
            p0 = torch.from_numpy(qvgen.seed_popularity(w.seed, w.n).astype(np.float32)).cuda()
        for name, fn in (("psgs", lambda: qv.qv_psgs(ctx0, g, w.fanouts)),
                         ("access_prob", lambda: qv.qv_access_prob(ctx0, g, w.fanouts, p0=p0))):
            fn()
            ctx0.sync()                                    # first call sizes the scratch arena
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(ctx0.stream)
            res = fn()
            e1.record(ctx0.stream)
            ctx0.sync()
            ms = e0.elapsed_time(e1)
            sweeps = len(w.fanouts) - 1 if name == "psgs" else len(w.fanouts)
            rp = rowptr.dtype.itemsize
            per_sweep = (w.n + 1) * rp + n_edges_graph * 8 + w.n * 8
            extra[name + "_ms"] = round(ms, 3)
            extra[name + "_algorithmic_GBps"] = round(max(sweeps, 1) * per_sweep / ms / 1e6, 1)
            if name == "access_prob":
                Pdev = res
            else:
                Qdev = res.clone()
        # FAP again with the in-edge CSR at hand (a symmetrised graph is its own transpose)
        t0 = time.perf_counter()
        g_in = g if w.symmetrise else g.transpose()
        if not w.symmetrise:
            extra["csr_transpose_ms"] = round((time.perf_counter() - t0) * 1e3, 1)
        qv.qv_access_prob(ctx0, g, w.fanouts, p0=p0, graph_in=g_in)
        ctx0.sync()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(ctx0.stream)
        P_in = qv.qv_access_prob(ctx0, g, w.fanouts, p0=p0, graph_in=g_in)
        e1.record(ctx0.stream)
        ctx0.sync()
        extra["access_prob_in_edge_form_ms"] = round(e0.elapsed_time(e1), 3)
        extra["access_prob_forms_max_rel_diff"] = float(((P_in - Pdev).abs() / Pdev.clamp_min(1e-30)).max().item())
        del g_in, P_in
        torch.cuda.empty_cache()
        log("psgs %.2f ms, access_prob %.2f ms (out-edges only) / %.2f ms (with the in-edge CSR) over the whole graph"
            % (extra["psgs_ms"], extra["access_prob_ms"], extra["access_prob_in_edge_form_ms"]))

    table_for_ablation = table if args.placement_ablation else None
    if tiered and not args.placement_ablation:
        if Pdev is None:
            Pdev = qv.qv_access_prob(ctx0, g, w.fanouts)
        rank = qv.qv_place_rank(ctx0, Pdev)
        ctx0.sync()
        feat = qv.Features(ctx0, table, hbm_budget_bytes=w.hbm_budget, rank=rank)
        del table
        torch.cuda.empty_cache()
        log("tiered features: %d of %d rows in HBM" % (feat.n_hot, w.n))
        hot_mask = torch.zeros(w.n, dtype=torch.bool, device="cuda")
        hot_mask[rank[:feat.n_hot].long()] = True
        # ceiling of the host link: pinned host -> device copy of 1 GiB
        pin = torch.empty(1 << 28, dtype=torch.int32, pin_memory=True)
        dst = torch.empty(1 << 28, dtype=torch.int32, device="cuda")
        dst.copy_(pin, non_blocking=True)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            dst.copy_(pin, non_blocking=True)
        e1.record()
        torch.cuda.synchronize()
        extra["host_link_pinned_copy_GBps"] = round(3 * pin.numel() * 4 / e0.elapsed_time(e1) / 1e6, 2)
        del pin, dst
    elif not args.placement_ablation:
        feat = qv.Features(ctx0, table, own_copy=True)     # rows re-laid on 128-byte boundaries where cheap
    else:
        feat = None

    if args.psgs_curve:
        return psgs_curve(qv, qvgen, w, ctx0, g, feat, Qdev, rowptr, col, tdtype)
    if args.placement_ablation:
        return placement_ablation(qv, qvgen, w, ctx0, g, table_for_ablation, Pdev, rowptr, col, tdtype)

    # ---- batches, contexts, buffers -------------------------------------------------------------
    # The timed region is a whole number of full calls (never a short call: --steps is rounded up to
    # calls of B batches), repeated until at least 50 ms have been timed; the median region gives
    # the figures.  Warm-up runs every timed batch once, so that nothing is touched for the first time
    # inside the region.
    import copy
    import math
    dedup_form = {"auto": 0, "table": 1, "partitioned": 2}[args.dedup]
    nb, eb, fb = qv.qv_sample_bounds(batch, w.fanouts, w.n)
    Kh = len(w.fanouts)
    L = qv.lib()
    # output rows are sized from what the batches really produce (the a-priori node bound is 15 x
    # larger on the citation workload); the sizes of every timed batch are checked against it below
    ctx0.set_dedup(dedup_form, args.partitions_log2)
    probe = [qv.qv_sample(ctx0, g, torch.from_numpy(w.seeds(b, batch)).cuda(), w.fanouts, w.rng_seed(b)) for b in range(4)]
    ctx0.sync()
    row_cap = min(nb, 2 * max(int(o.node_off[-1].item()) for o in probe) + 1024)
    del probe
    # batches per call: as asked, unless one call's buffers (outputs at their a-priori bounds, scratch of
    # about the same size, gathered rows) would not fit beside the graph and the feature table
    B = max(1, min(args.batches_per_call, qv.QV_MAX_BATCHES))
    per_batch_bytes = 2 * (eb * 8 + nb * 4) + row_cap * feat.row_stride
    free_bytes = torch.cuda.mem_get_info()[0]
    while B > 8 and B * per_batch_bytes > 0.6 * free_bytes:
        B //= 2
    if B != args.batches_per_call:
        log("%d batches per call (%.1f GB of buffers per call, %.0f GB free)" % (B, B * per_batch_bytes / 1e9, free_bytes / 1e9))
    calls_per_region = max(1, math.ceil(K / B))
    calls_per_region = math.ceil(calls_per_region / S) * S          # every stream gets the same number of calls
    n_batches = calls_per_region * B
    seeds_host = [w.seeds(b, batch) for b in range(n_batches)]
    seeds_dev = [torch.from_numpy(s).cuda() for s in seeds_host]
    rng_seeds = [w.rng_seed(b) for b in range(n_batches)]

    made_contexts = []

    def new_context(stream):
        c = qv.Context(0, stream)
        made_contexts.append(c)
        if args.table_budget_gib >= 0:
            c.set_table_budget(int(args.table_budget_gib * 2 ** 30))
        c.set_dedup(dedup_form, args.partitions_log2)
        c.reserve(batch, w.fanouts, w.n, n_batches=B)
        return c

    class Lane:
        """One context (stream) with the buffers of one call."""
        def __init__(self, ctx):
            self.ctx = ctx
            self.bufs = [qv.SampleBuffers(ctx, batch, w.fanouts, w.n, want_frontier=False, want_nbr_global=False)
                         for _ in range(B)]
            self.rows = [feat.empty_rows(row_cap, "cuda") for _ in range(B)]
            self.plan = qv.ManyPlan(ctx, g, feat, self.bufs, self.rows, w.fanouts)
            for t in range(B):
                self.plan.n_ids[t] = row_cap

    lanes = [Lane(ctx0 if i == 0 else new_context(torch.cuda.Stream())) for i in range(S)]
    if S >= 1:
        if args.table_budget_gib >= 0:
            ctx0.set_table_budget(int(args.table_budget_gib * 2 ** 30))
        ctx0.reserve(batch, w.fanouts, w.n, n_batches=B)
    # per-batch size blocks so that counts can be read after the timed region
    offs = [(torch.zeros(Kh + 2, dtype=torch.int64, device="cuda"), torch.zeros(Kh + 1, dtype=torch.int64, device="cuda"),
             torch.zeros(Kh + 2, dtype=torch.int64, device="cuda")) for _ in range(n_batches)]

    plan_cache = {}

    def plan_for(lane, j):
        """Argument arrays of call j (batches j*B .. j*B+B-1) on this lane, marshalled once."""
        key = (id(lane), j)
        p = plan_cache.get(key)
        if p is None:
            views = []
            for t in range(B):
                v = copy.copy(lane.bufs[t])
                v.node_off, v.edge_off, v.frontier_off = offs[j * B + t]
                views.append(v)
            p = qv.ManyPlan(lane.ctx, g, feat, views, lane.rows, w.fanouts)
            for t in range(B):
                p.n_ids[t] = row_cap
                p.seed_ptrs[t] = seeds_dev[j * B + t].data_ptr()
                p.n_seeds[t] = batch
                p.rng[t] = rng_seeds[j * B + t]
            plan_cache[key] = p
        return p

    def issue(lane, j, events=None):
        """One full call: the B batches of call j through sampling and gather."""
        p, c = plan_for(lane, j), lane.ctx
        if events:
            events[0].record(c.stream)
        c.check(L.qv_sample_many(c.h, g.h, B, p.seed_ptrs, p.n_seeds, p.fan, p.k, p.rng, 0, p.outs))
        if events:
            events[1].record(c.stream)
        c.check(L.qv_gather_many(c.h, feat.h, B, p.ids, p.n_ids, p.n_dev, p.out_ptrs, p.stride))
        if events:
            events[2].record(c.stream)

    def region(lns, timed_events=None, n_calls=None):
        n_calls = n_calls or calls_per_region
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for j in range(n_calls):
            issue(lns[j % len(lns)], j % calls_per_region, timed_events[j] if timed_events else None)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def measure(lns, min_seconds, min_regions, with_events, n_calls=None):
        times, evs = [], []
        for _ in range(max(2, math.ceil(W / max(1, n_batches)))):      # warm-up: whole regions
            region(lns, None, n_calls)
        while (sum(times) < min_seconds or len(times) < min_regions) and len(times) < 400:
            e = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(calls_per_region)] if with_events else None
            times.append(region(lns, e, n_calls))
            if e:
                evs.append(e)
        for ln in lns:
            ln.ctx.sync()                                      # raises on a deferred device error
        return times, evs

    region_s, region_ev = measure(lanes, 0.05, 5, True)
    elapsed = float(np.median(region_s))                       # seconds per region of n_batches steps

    # ---- the same region over other stream counts (reported beside the main figure) --------------
    # With one stream every kernel's duration is its own, which is what the roofline entry needs;
    # several contexts on their own streams let calls overlap (the paper's multiplexed pipelines).
    sweep = {}
    sweep_note = None
    if args.extra_streams > 0 and not tiered and S == 1:
        sweep_lanes = list(lanes)
        for S2 in (1, 2, 4, 8, 16):
            if S2 > args.extra_streams:
                continue
            try:
                while len(sweep_lanes) < S2:
                    sweep_lanes.append(Lane(new_context(torch.cuda.Stream())))
            except (qv.QvError, torch.OutOfMemoryError) as e:   # every context holds scratch for a whole call
                sweep_note = "stopped before %d streams: %s" % (S2, str(e)[:120])
                log("stream sweep " + sweep_note)
                break
            n_calls = max(calls_per_region, 2 * S2)            # at least two calls per stream in flight
            ts, _ = measure(sweep_lanes[:S2], 0.03, 3, False, n_calls)
            sweep[str(S2)] = round(float(np.median(ts)) * 1e3 / (n_calls * B), 5)
        # give the extra contexts' scratch and buffers back before the passes below
        torch.cuda.synchronize()
        plan_cache = {k: v for k, v in plan_cache.items() if k[0] in {id(ln) for ln in lanes}}
        for ln in sweep_lanes[len(lanes):]:
            ln.plan = None
            ln.bufs = ln.rows = None
            ln.ctx.close()
        del sweep_lanes
        import gc
        gc.collect()
        torch.cuda.empty_cache()

    # ---- the same batches through qv_step_many, four groups of B on the library's own streams ----
    step_ms = None
    if args.extra_streams > 0 and not tiered and S == 1 and B == qv.QV_MAX_BATCHES:
        nS = qv.QV_MAX_STEP_BATCHES
        try:
            s_bufs = lanes[0].bufs + [qv.SampleBuffers(ctx0, batch, w.fanouts, w.n, want_frontier=False, want_nbr_global=False)
                                      for _ in range(nS - B)]
            s_rows = lanes[0].rows + [feat.empty_rows(row_cap, "cuda") for _ in range(nS - B)]
            s_plan = qv.ManyPlan(ctx0, g, feat, s_bufs, s_rows, w.fanouts)
            for t in range(nS):
                s_plan.n_ids[t] = row_cap
            s_seeds = [seeds_dev[t % n_batches] for t in range(nS)]
            s_rng = [rng_seeds[t % n_batches] for t in range(nS)]
            ts = []
            for rep in range(2 + 7):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                s_plan.step(s_seeds, s_rng)
                s_plan.step(s_seeds, s_rng)
                torch.cuda.synchronize()
                if rep >= 2:
                    ts.append((time.perf_counter() - t0) / 2)
            ctx0.sync()
            step_ms = float(np.median(ts)) * 1e3 / nS
            del s_plan, s_bufs, s_rows
        except (qv.QvError, torch.OutOfMemoryError) as e:
            log("qv_step_many pass skipped: " + str(e)[:120])
        import gc
        gc.collect()
        torch.cuda.empty_cache()

    # ---- latency pass (not part of the timed region): one batch per call, one at a time ---------
    n_lat = max(220, args.latency_samples + 20)
    lat_plan = qv.ManyPlan(ctx0, g, feat, [lanes[0].bufs[0]], [lanes[0].rows[0]], w.fanouts)
    lat_plan.n_ids[0] = row_cap
    lat_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_lat)]
    for i in range(n_lat):
        lat_ev[i][0].record(ctx0.stream)
        lat_plan.run([seeds_dev[i % n_batches]], [rng_seeds[i % n_batches]])
        lat_ev[i][1].record(ctx0.stream)
        ctx0.sync()
    lat_ms = [a.elapsed_time(b) for a, b in lat_ev[20:]]

    # ---- accounting (one region) ---------------------------------------------------------------
    tot_edges = tot_unique = tot_front = 0
    samp_b = reidx_b = gath_b = 0
    if Qdev is not None:        # PSGS summed over a batch's seeds: the predicted size of its sampled tree
        sums = [qv.qv_psgs_batch_sum(ctx0, Qdev, seeds_dev[i]) for i in range(min(n_batches, 32))]
        ctx0.sync()
        extra["psgs_sum_per_batch"] = round(float(np.mean([x.item() for x in sums])), 1)
    max_unique = 0
    for i in range(n_batches):
        no, eo, fo = (t.cpu().numpy() for t in offs[i])
        U, E, F = int(no[-1]), int(eo[-1]), int(fo[Kh])        # frontier entries expanded = F_0..F_{K-1}
        max_unique = max(max_unique, U)
        tot_edges += E
        tot_unique += U
        tot_front += F
        sb, rb, gb = algorithmic_bytes(F, E, U, U, w.row_bytes, rowptr.dtype.itemsize, tiered)
        samp_b += sb
        reidx_b += rb
        gath_b += gb
    assert max_unique <= row_cap, "a batch produced more distinct nodes (%d) than the output rows hold (%d)" % (max_unique, row_cap)
    if tiered:                  # rows of the last call's batches that came over the host link
        cold = tot = 0
        last = lanes[(calls_per_region - 1) % S]
        for t in range(B):
            U = int(offs[(calls_per_region - 1) * B + t][0][-1].item())
            ids = last.bufs[t].n_id[:U].long()
            cold += int((~hot_mask[ids]).sum().item())
            tot += U
        extra["cold_row_fraction"] = round(cold / max(tot, 1), 4)
    sample_ms = [e[0].elapsed_time(e[1]) for reg in region_ev for e in reg]
    gather_ms = [e[1].elapsed_time(e[2]) for reg in region_ev for e in reg]
    batch_ms = [e[0].elapsed_time(e[2]) for reg in region_ev for e in reg]
    ms_per_step = elapsed * 1e3 / n_batches
    # a qv_gather_many call issues its id lists GATHER_LISTS_PER_LAUNCH to a k_gather launch, back to back
    launches_per_call = (B + GATHER_LISTS_PER_LAUNCH - 1) // GATHER_LISTS_PER_LAUNCH
    gather_call_ms = float(np.mean(gather_ms))
    gather_avg_ms = gather_call_ms / launches_per_call
    gather_bytes_per_launch = gath_b / calls_per_region / launches_per_call
    achieved = gather_bytes_per_launch / (gather_avg_ms * 1e-3) / 1e9
    path_bytes = samp_b + reidx_b + gath_b
    ratio = GATHER_TRAFFIC_RATIO.get((w.name, args.scale, min(B, GATHER_LISTS_PER_LAUNCH)))

    result = {
        "metric": "sampled_edges_per_s",
        "value": round(tot_edges / elapsed, 1),
        "unit": "edges/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32",       # ids, offsets and counters; feature rows are copied bit for bit
        "data": "synthetic",
        "config": {"workload": "%s: %d nodes, %d edges, %s x %d features, fanouts %s, batch %d%s" %
                   (w.name, w.n, n_edges_graph, "fp16" if tdtype == torch.float16 else "fp32", w.dim, w.fanouts,
                    batch, ", %d rows in HBM / rest host-pinned" % feat.n_hot if tiered else ", features all in HBM"),
                   "streams": S, "batches_per_call": B, "scale": args.scale, "dedup": args.dedup},
        "timed": {"steps_per_region": n_batches, "calls_per_region": calls_per_region, "regions": len(region_s),
                  "region_ms_median": round(elapsed * 1e3, 4), "region_ms_min": round(min(region_s) * 1e3, 4),
                  "region_ms_max": round(max(region_s) * 1e3, 4), "timed_seconds": round(sum(region_s), 4),
                  "note": "--steps is rounded up to whole calls of batches_per_call; the region is repeated until 50 ms "
                          "have been timed and the median region is reported"},
        "sampled_edges_per_batch": round(tot_edges / n_batches, 1),
        "unique_nodes_per_batch": round(tot_unique / n_batches, 1),
        "gathered_feature_GBps": round(tot_unique * w.row_bytes / calls_per_region / (gather_call_ms * 1e-3) / 1e9, 2),
        "gather_frac_hbm_peak": round(achieved / HBM_PEAK_GBPS, 4),
        "path_algorithmic_GBps": round(path_bytes / elapsed / 1e9, 2),
        "path_frac_hbm_peak": round(path_bytes / elapsed / 1e9 / HBM_PEAK_GBPS, 4),
        "p50_batch_latency_ms": round(float(np.percentile(lat_ms, 50)), 4),
        "p99_batch_latency_ms": round(float(np.percentile(lat_ms, 99)), 4),
        "latency_samples": len(lat_ms),
        "p50_call_latency_ms": round(float(np.percentile(batch_ms, 50)), 4),
        "sample_ms_avg": round(float(np.mean(sample_ms)), 4),
        "gather_ms_avg": round(gather_call_ms, 4),
        "roofline": {"bound": "hbm", "kernel": "k_gather", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": round(ratio * gather_bytes_per_launch) if ratio else None,
                     "traffic_source": (GATHER_TRAFFIC_PROFILE if ratio else
                                        "no rocprofv3 counter run is committed for this workload and batches per call"),
                     "bytes_per_launch": round(gather_bytes_per_launch), "avg_launch_ms": round(gather_avg_ms, 5),
                     "launches_timed": len(gather_ms) * launches_per_call, "lists_per_launch": min(B, GATHER_LISTS_PER_LAUNCH)},
    }
    if tiered:
        cold_bytes = extra["cold_row_fraction"] * tot_unique * w.row_bytes
        extra["cold_tier_GBps"] = round(cold_bytes / calls_per_region / (gather_call_ms * 1e-3) / 1e9, 2)
        result["roofline"]["note"] = ("tiered: %.0f%% of the rows come over the host link, which bounds this "
                                      "kernel, not HBM" % (100 * extra["cold_row_fraction"]))
    if sweep:
        extra["stream_sweep"] = {"batches_per_call": B, "ms_per_step_by_streams": sweep,
                                 "best_path_frac_hbm_peak": round(path_bytes / n_batches / (min(sweep.values()) * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                 "best_value": round(tot_edges / n_batches / (min(sweep.values()) * 1e-3), 1)}
        if sweep_note:
            extra["stream_sweep"]["note"] = sweep_note
        best_s = min(sweep, key=sweep.get)
        extra["best_sustained"] = {"streams": int(best_s), "value": extra["stream_sweep"]["best_value"], "unit": "edges/s",
                                   "ms_per_step": sweep[best_s],
                                   "path_frac_hbm_peak": extra["stream_sweep"]["best_path_frac_hbm_peak"],
                                   "note": "best of the stream sweep (whole calls of batches_per_call on each stream); `value` above is the "
                                           "one-stream figure, where a kernel's duration is its own"}
    if step_ms:
        extra["step_many"] = {"batches_per_call": qv.QV_MAX_STEP_BATCHES, "ms_per_step": round(step_ms, 5),
                              "value": round(tot_edges / n_batches / (step_ms * 1e-3), 1), "unit": "edges/s",
                              "path_frac_hbm_peak": round(path_bytes / n_batches / (step_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                              "note": "one context, qv_step_many: four groups of %d batches, three of them on the library's own streams" % B}
    result.update(extra)

    # ---- the oracle on this machine's host cores (a reported baseline, not the target) ------------
    if not args.no_cpu_baseline:
        import oracle
        from concurrent.futures import ThreadPoolExecutor
        sub_rows = min(w.n, 4_000_000)
        host_table = qvgen.features_host(w.seed, sub_rows, w.dim, w.feat_dtype)

        def one(i):
            t1 = time.perf_counter()
            o = oracle.sample(rowptr, col, seeds_host[i % n_batches], w.fanouts, rng_seeds[i % n_batches])
            oracle.gather(host_table, o["n_id"] % sub_rows)
            return time.perf_counter() - t1, int(o["edge_off"][-1])

        t_budget, t_used, e_cpu, nb_cpu = 10.0, 0.0, 0, 0
        while t_used < t_budget and nb_cpu < 4 * n_batches:
            dt, e = one(nb_cpu)
            t_used += dt; e_cpu += e; nb_cpu += 1
        result["cpu_baseline"] = {
            "value": round(e_cpu / t_used, 1), "unit": "edges/s", "cores": 1, "kind": "oracle",
            "sample": "%d batches of the timed workload, single-threaded oracle sample+reindex+gather; gather rows taken "
                      "modulo a %d-row host table" % (nb_cpu, sub_rows),
            "ms_per_batch": round(t_used * 1e3 / nb_cpu, 3)}
        # the same oracle, one independent batch per thread on T threads (the oracle releases the interpreter lock)
        T = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")), 16))
        per_thread = max(1, int(10.0 / (t_used / nb_cpu) / 1.0))
        per_thread = min(per_thread, 64)
        t1 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=T) as pool:
            res = list(pool.map(lambda th: sum(one(th * per_thread + j)[1] for j in range(per_thread)), range(T)))
        t_mt = time.perf_counter() - t1
        result["cpu_baseline_threads"] = {
            "value": round(sum(res) / t_mt, 1), "unit": "edges/s", "cores": T, "kind": "oracle",
            "sample": "%d threads x %d batches each, the unmodified single-threaded oracle on independent batches" % (T, per_thread),
            "seconds": round(t_mt, 2)}
    import subprocess
    try:
        result["git"] = subprocess.check_output(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], stderr=subprocess.DEVNULL).decode().strip()
    except Exception:
        try:        # a copy of the tree without history: the commit the library was built from
            with open(os.path.join(ROOT, "paper_2305_10863_amd", "build_info.json")) as f:
                info = json.load(f)
            result["git"] = None if info.get("git") is None else info["git"] + (" (built from a modified tree)" if info.get("dirty") else "")
        except Exception:
            result["git"] = None
    line = json.dumps(result)
    try:
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "bench_%s.json" % w.name), "w") as f:
            f.write(line + "\n")
    except OSError:
        pass
    print(line, flush=True)
    # handles go before the interpreter starts tearing the GPU runtime down
    torch.cuda.synchronize()
    plan_cache.clear()
    feat.close()
    for c in made_contexts:
        c.close()
    g.__del__()
    ctx0.close()


if __name__ == "__main__":
    main()
