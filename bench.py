#!/usr/bin/env python3
"""Benchmark of the packed multi-field embedding step (forward + backward +
sparse Adagrad) on one MI355X.

A "step" is one pass of the whole hot path over one batch: pk_forward followed
by pk_backward_update.  Inputs (IDs, offsets, gradients) and tables are
synthetic, seeded, and resident in HBM before the timed region; a ring of
distinct batches is cycled so that no step sees the batch of the step before.
Prints ONE JSON line.  With no --workload it times the 26-field configuration
(the headline figures of the line) and the 200-field configuration (the same
figures under "workloads"), one after the other.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def algorithmic_bytes(info, mean_pack):
    """Bytes each kernel must move for one pack with measured sizes
    (nnz, U, k*B bags, dim D, element size sw, bitmap bytes bm).  Rows are
    counted once per DISTINCT key: removing repeats is the method."""
    n, U, bags, D, sw, bm = info["nnz"], info["U"], info["bags"], info["D"], info["sw"], info["bitmap_bytes"]
    ent = 4 * n + sc_occ(n, mean_pack)                      # the occurrences grouped by key (with bag lengths for mean pooling)
    return {
        # small batches, the forward pass in one launch: ids and offsets in; keys, inverse, grouped occurrences,
        # distinct keys, segment offsets and packed offsets out; one read of each distinct row; pooled output
        "pk_fused": 8 * n + 4 * bags + 4 * n + 4 * n + ent + 8 * U + 4 * bags + sw * D * U + 4 * D * bags,
        "pk_keys": 8 * n + 4 * n + 4 * bags + 4 * bags,
        "pk_pool": 4 * n + 4 * (bags + 1) + sw * D * U + 4 * D * bags,
        "pk_scatter": 4 * n + 4 * bags + 8 * n,
        "pk_slices_mark": 8 * n + bm,        # (the listed slices' launches, pk_slices_*_big, share these bytes)
        "pk_slices_place": 8 * n + bm + ent + 8 * U + bm // 8,
        "pk_inverse": 8 * n + min(bm + bm // 8, 36 * n),
        "pk_adagrad": 4 * (U + 1) + 4 * U + ent + 4 * D * bags + (2 * sw + 8) * D * U,
    }


def sc_occ(n, mean_pack):
    """bytes of the per-occurrence 1/L scales (only packs with mean pooling carry them)"""
    return 4 * n if mean_pack else 0


def step_model_bytes(info):
    """Whole-step algorithmic traffic of one pack: ids, offsets, one read of each
    distinct row, output write, gradient read, W and A read+write per distinct
    row, inverse write+read, unique write+read."""
    n, U, bags, D, sw = info["nnz"], info["U"], info["bags"], info["D"], info["sw"]
    return (8 * n + 4 * (bags + 1) + sw * D * U + 4 * D * bags + 4 * D * bags + (2 * sw + 8) * D * U
            + 8 * n + 8 * U)


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` as rocprofv3's FETCH_SIZE / WRITE_SIZE counters measured them on this
    workload (two --pmc runs of this script, scaled by what the same counters read for a plain 1 GiB copy);
    the summary under profiles/ holds the per-kernel figures and the commands.  None when it is not there."""
    path = os.path.join(ROOT, "profiles", f"all_kernels_{workload}_hbm_traffic.txt")
    totals = []
    try:
        with open(path) as fh:
            for line in fh:
                name = line.split(" ")[0]
                if name == kernel + "_kernel" or name.startswith(kernel + "_kernel<"):
                    totals.append(float(line.split("total=")[1]) * 1e6)      # MB per launch
    except OSError:
        pass
    rel = os.path.relpath(path, ROOT)
    return (sum(totals) / len(totals), rel) if totals else (None, None)   # one launch of each instantiation per step


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=None, choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"],
                    help="one workload only (default: cfg2 as the headline and cfg3 beside it)")
    ap.add_argument("--ring", type=int, default=0, help="distinct batches cycled (default 16, 4 for cfg3-5)")
    ap.add_argument("--max-shards", type=int, default=0,
                    help="Eq. 1 shard split of heavy packs (0 = off, the configurations' own pack counts); the "
                         "per-field occurrence counts of the first batch serve as the warm-up statistics")
    ap.add_argument("--groups", type=int, default=0,
                    help="K-Interleaving groups of packed operations (0 = chosen by batch size, 1 = none)")
    ap.add_argument("--hot-fraction", type=float, default=None,
                    help="HybridHash: keep this fraction of every pack's rows in a device Hot-storage in front of "
                         "the tables (Cold-storage); reports the hit ratio of the batches' distinct rows")
    ap.add_argument("--cold", default="host", choices=["host", "device"],
                    help="HybridHash: where the Cold-storage lives (pinned host memory or device memory)")
    ap.add_argument("--hh-warmup", type=int, default=20)
    ap.add_argument("--hh-flush", type=int, default=10)
    ap.add_argument("--micro-batches", type=int, default=0,
                    help="D-Interleaving: cut every batch into this many micro-batches and pass them through the "
                         "layer one after the other, the next one's dedup on a second stream (1 = whole batches, "
                         "pipelined the same way; 0 = off: one pk_forward and one pk_backward_update per batch)")
    ap.add_argument("--micro-serial", action="store_true",
                    help="with --micro-batches: no second stream, every micro-batch starts when the one before is done")
    ap.add_argument("--partition", type=int, default=0,
                    help="also time Partition (Sec. II-D) of every pack's distinct keys over this many owners, after "
                         "the timed steps, and report the sizes of the owners' groups and what Shuffle would carry")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a known size for scaling rocprofv3's byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only; run it with --gpus 1 (no collectives or sharding are "
              "part of it)", file=sys.stderr)
        sys.exit(2)
    return args


def run_workload(args, workload):
    """Times one workload; returns the result dictionary (the JSON line's fields)."""
    import numpy as np
    import torch

    import synth
    from paper_2204_04903_amd import binding as pk
    from paper_2204_04903_amd.layer import HybridEmbedding, MicroBatchPipeline, PackedEmbedding

    idx = int(workload[3])
    wl = synth.config(idx)
    ring = args.ring or (16 if idx <= 2 else 4)
    tables = [(t.rows, t.dim, t.dtype) for t in wl.tables]
    fields = [(f.table, f.pool) for f in wl.fields]
    t0 = time.time()
    batches = synth.make_batches(wl, ring)
    gen_s = time.time() - t0

    torch.cuda.set_device(0)
    plan_opts = {}
    if args.max_shards > 1:
        b0 = batches[0]
        plan_opts = dict(max_shards=args.max_shards,
                         field_volume=[float(b0.offsets[(f + 1) * wl.batch] - b0.offsets[f * wl.batch])
                                       for f in range(wl.n_fields)])
    if args.groups:
        plan_opts["interleave_groups"] = args.groups
    hybrid = args.hot_fraction is not None
    if hybrid:
        probe = pk.pk_plan_create(tables, fields, **plan_opts)
        hot_rows = [int(pk.pk_plan_pack_info(probe, p)["total_rows"] * args.hot_fraction)
                    for p in range(pk.pk_plan_num_packs(probe))]
        pk.pk_plan_destroy(probe)
        layer = HybridEmbedding(tables, fields, hot_rows, args.hh_warmup, args.hh_flush,
                                cold_on_host=args.cold == "host", **plan_opts)
    else:
        layer = PackedEmbedding(tables, fields, **plan_opts)
    stream = torch.cuda.current_stream().cuda_stream
    for t, ts in enumerate(wl.tables):
        synth.fill_device(layer.table_view(t).data_ptr(), ts.rows, ts.dim, ts.dtype, wl.seed, t, stream)
    dev = [(torch.from_numpy(b.ids).cuda(), torch.from_numpy(b.offsets).cuda(), torch.from_numpy(b.grad_out).cuda())
           for b in batches]
    max_nnz = max(b.nnz for b in batches)
    layer._ensure_ws(wl.batch, max_nnz)
    out = torch.empty((wl.batch, layer.out_dim), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def step(i):
        ids, offsets, grad = dev[i % ring]
        layer.forward(ids, offsets, wl.batch, out=out)
        layer.backward_update(grad, wl.lr, wl.eps)
        if hybrid:
            layer.end_iteration(want_counts=False)

    micro_info = None
    if args.micro_batches > 0 and not hybrid:
        # the ring's batches cut into micro-batches, resident like the whole batches
        M = args.micro_batches
        mdev = []
        for b in batches:
            row = []
            for mb in synth.split_batch(b, wl.n_fields, wl.batch, M):
                row.append((torch.from_numpy(mb.ids).cuda(), torch.from_numpy(mb.offsets).cuda(),
                            torch.from_numpy(mb.grad_out).cuda(), mb.grad_out.shape[0]))
            mdev.append(row)
        b_max = max(m[3] for row in mdev for m in row)
        n_max = max(int(m[0].shape[0]) for row in mdev for m in row)
        pipe = MicroBatchPipeline(layer, b_max, n_max)
        bounds = [(wl.batch * m) // M for m in range(M + 1)]

        def run_steps(first, count):
            seq = [((first + i) % ring, m) for i in range(count) for m in range(M)]
            if args.micro_serial:
                for r, m in seq:
                    ids, offsets, grad, bm = mdev[r][m]
                    t = pipe.submit(ids, offsets, bm)
                    pipe.pool(t, out[bounds[m]:bounds[m + 1]])
                    pipe.backward_update(t, grad, wl.lr, wl.eps)
                return
            t = pipe.submit(*mdev[seq[0][0]][seq[0][1]][:2], mdev[seq[0][0]][seq[0][1]][3])
            for j, (r, m) in enumerate(seq):
                nxt = None
                if j + 1 < len(seq):
                    ids, offsets, _, bm = mdev[seq[j + 1][0]][seq[j + 1][1]]
                    nxt = pipe.submit(ids, offsets, bm)
                pipe.pool(t, out[bounds[m]:bounds[m + 1]])
                pipe.backward_update(t, mdev[r][m][2], wl.lr, wl.eps)
                t = nxt

        micro_info = {"micro_batches": M, "micro_batch_size": b_max, "interleaved": not args.micro_serial,
                      "workspace_bytes": 2 * pipe.ws_bytes,
                      "whole_batch_workspace_bytes": pk.pk_workspace_bytes(layer.plan, wl.batch, max_nnz)}
    else:
        def run_steps(first, count):
            for i in range(count):
                step(first + i)

    if hybrid:                       # Alg. 1's warm-up iterations and the first reload come before the clock
        args.warmup = max(args.warmup, args.hh_warmup + args.hh_flush + 1)
    run_steps(0, args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(args.warmup, args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    lookups = sum(batches[(args.warmup + i) % ring].nnz for i in range(args.steps))
    ms_per_step = elapsed * 1e3 / args.steps
    value = lookups / elapsed

    hybrid_info = None
    if hybrid:                       # hit ratio of the distinct rows of a batch, over one pass of the ring
        q_tot = h_tot = 0
        for i in range(ring):
            ids, offsets, grad = dev[i % ring]
            layer.forward(ids, offsets, wl.batch, out=out)
            layer.backward_update(grad, wl.lr, wl.eps)
            q, h, _ = layer.end_iteration(want_counts=True)
            q_tot += sum(q); h_tot += sum(h)
        hybrid_info = {"hot_fraction": args.hot_fraction, "cold_storage": args.cold, "warmup_iters": args.hh_warmup,
                       "flush_iters": args.hh_flush, "hit_ratio": h_tot / max(1, q_tot),
                       "hot_rows": [layer.hot_count(p) for p in range(layer.n_packs)]}

    # ---- per-kernel durations (HIP events on the launch stream) and sizes --------------------
    prof_steps = min(args.steps, 4 * ring)
    pk.pk_profile_enable(layer.plan, True)
    sizes = []                      # per profiled step, per pack
    for i in range(prof_steps):
        step(i)
        row = []
        for p in range(layer.n_packs):
            d = pk.pk_ctx_pack(layer.plan, layer.ws, wl.batch, batches[i % ring].nnz, p)
            info = layer.packs[p]
            row.append(dict(nnz=d["nnz_p"], U=d["n_unique"], bags=info["n_fields"] * wl.batch, D=info["dim"],
                            sw=4 if info["dtype"] == 0 else 2, bitmap_bytes=(info["total_rows"] + 7) // 8))
        sizes.append(row)
    prof = pk.pk_profile_read(layer.plan)
    pk.pk_profile_enable(layer.plan, False)
    mean_pack = [any(fields[f][1] == 1 for f in layer.pack_fields[p]) for p in range(layer.n_packs)]
    kern = {}
    for name, (ms, launches) in prof.items():
        kern[name] = dict(ms_per_step=ms / prof_steps, launches_per_step=launches / prof_steps)
    alg = {}
    for row in sizes:
        for p, info in enumerate(row):
            for k, v in algorithmic_bytes(info, mean_pack[p]).items():
                alg[k] = alg.get(k, 0) + v
    model_bytes = sum(step_model_bytes(info) for row in sizes for info in row) / prof_steps
    for k in kern:
        if k in alg:
            kern[k]["alg_bytes_per_step"] = alg[k] / prof_steps
            kern[k]["GBps"] = alg[k] / prof_steps / (kern[k]["ms_per_step"] * 1e-3) / 1e9
    # the dominant kernel is the one that takes the most time, nothing else; the kernels within 5 % of it
    # are listed beside it with their own figures
    dom = max(kern, key=lambda k: kern[k]["ms_per_step"])
    t_max = kern[dom]["ms_per_step"]
    dk = kern[dom]
    launches = max(1.0, dk["launches_per_step"])
    traffic, traffic_file = measured_traffic(dom, workload)
    roofline = {
        "kernel": dom,
        "bound": "hbm",
        "achieved": dk.get("GBps"),
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": (dk["GBps"] / HBM_PEAK_GBPS) if "GBps" in dk else None,
        "traffic": traffic,
        "traffic_source": (f"{traffic_file}: rocprofv3 --pmc runs of this command, kept as a file; not measured "
                           f"in this run") if traffic is not None else None,
        "alg_bytes_per_launch": dk.get("alg_bytes_per_step", 0) / launches,
        "avg_launch_ms": dk["ms_per_step"] / launches,
        "within_5pct": {k: {"avg_launch_ms": v["ms_per_step"] / max(1.0, v["launches_per_step"]),
                            "frac": v["GBps"] / HBM_PEAK_GBPS if "GBps" in v else None}
                        for k, v in kern.items() if k != dom and v["ms_per_step"] >= 0.95 * t_max},
        "whole_step_frac": model_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
    }
    torch.cuda.synchronize()
    if layer.error_word() != 0:
        raise RuntimeError(f"{workload}: the device error word is {layer.error_word()} after the timed steps")

    # ---- Partition of the last step's distinct keys (outside the timed steps) ----------------------
    partition_info = None
    if args.partition > 0 and not hybrid:
        n_own = args.partition
        reps = 20
        step(0)
        for p in range(layer.n_packs):
            layer.partition(p, n_own)                                   # warm-up
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        nnz0 = batches[0].nnz
        need = pk.pk_partition_scratch_bytes(layer.plan, nnz0, n_own)
        scratch = torch.empty(need, dtype=torch.uint8, device="cuda")
        pkeys = torch.empty(nnz0, dtype=torch.int32, device="cuda")
        pidx = torch.empty(nnz0, dtype=torch.int32, device="cuda")
        poffs = [torch.empty(n_own + 1, dtype=torch.int32, device="cuda") for _ in range(layer.n_packs)]
        e0.record()
        for _ in range(reps):
            for p in range(layer.n_packs):
                pk.pk_partition_unique(layer.plan, layer.ws, layer.ws_bytes, wl.batch, nnz0, p, n_own, pkeys, pidx,
                                       poffs[p], scratch, need, stream)
        e1.record()
        torch.cuda.synchronize()
        packs = []
        for p in range(layer.n_packs):
            o = poffs[p].cpu().numpy().astype(np.int64)
            cnt = np.diff(o)
            info = layer.packs[p]
            row_b = info["dim"] * (4 if info["dtype"] == 0 else 2)
            away = int(cnt.sum() - cnt[0])                             # this worker is owner 0: the rest travels
            packs.append({"distinct_keys": int(o[-1]), "per_owner": cnt.tolist(),
                          "keys_sent_bytes": 4 * away, "rows_received_bytes": row_b * away,
                          "gradient_rows_sent_bytes": 4 * info["dim"] * away})
        tot = sum(q["keys_sent_bytes"] + q["rows_received_bytes"] + q["gradient_rows_sent_bytes"] for q in packs)
        partition_info = {"owners": n_own, "rule": "row mod owners", "ms_per_step": e0.elapsed_time(e1) / reps,
                          "alg_bytes_per_step": sum(12 * q["distinct_keys"] for q in packs),
                          "packs": packs, "shuffle_bytes_per_step": tot,
                          "shuffle_bytes_per_link": tot / max(1, n_own - 1)}

    # ---- the CPU oracle on the host cores, bounded samples --------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(workload, wl, batches, ring, synth)

    result = {
        "metric": "pooled embedding lookups/sec (fwd+bwd+update)",
        "value": value,
        "unit": "lookups/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if wl.tables[0].dtype == 0 else "bf16 tables, f32 arithmetic",
        "data": "synthetic",
        "config": {"workload": f"{workload}: {wl.description}" + (" [HybridHash]" if hybrid else "") + (f" [{args.micro_batches} micro-batch(es) per batch]" if micro_info else ""), "batch": wl.batch, "fields": wl.n_fields,
                   "packs": layer.n_packs, "max_shards": args.max_shards, "interleave_groups": args.groups, "ring_batches": ring, "lookups_per_step": lookups / args.steps,
                   "distinct_keys_per_step": sum(i["U"] for i in sizes[0])},
        "hbm_model": {"bytes_per_step": model_bytes, "GBps": model_bytes / (ms_per_step * 1e-3) / 1e9,
                      "frac_of_peak": model_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "hybrid_hash": hybrid_info,
        "d_interleaving": micro_info,
        "partition": partition_info,
        "kernels": {k: {kk: round(vv, 6) for kk, vv in v.items()} for k, v in kern.items()},
        "input_generation_s": round(gen_s, 2),
    }
    layer.close()
    del layer, dev, out
    torch.cuda.empty_cache()
    return result


def cpu_baseline(workload, wl, batches, ring, synth, budget_s=8.0):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same batches.
    Two figures: (i) the parity oracle itself, one thread, whole packs; (ii) the same step functions over
    independent units, one table and its fields each (tables share no rows and no output columns), handed to a
    pool of threads, one per core of the box's share.  `value` is (ii); (i) is under "single_thread".  The rows
    of the distinct keys are materialised by the input generator, and the per-table inputs are cut out of the
    batch, before the clock starts (staging, like the copy of the inputs to the device)."""
    import copy
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    from oracle import pk_oracle as orc
    from oracle.sparse_tables import SparseOracle

    host_cores = os.cpu_count() or 1
    threads = max(1, min(16, host_cores))        # a one-GPU machine's share of the host is 16 cores
    so = SparseOracle(orc, synth, wl)
    times, looks, n_cpu = [], 0, 0
    while sum(times) < budget_s and n_cpu < 4 * ring:
        b = batches[n_cpu % ring]
        pre = []
        for p in range(so.pl.n_packs):
            key, _ = orc.pack_keys(so.pl, p, wl.batch, b.ids, b.offsets)
            uq, _ = orc.unique(key)
            pre.append(so.current_rows(p, uq))
        t1 = time.perf_counter()
        so.step(b, wl.lr, wl.eps, rows=pre)
        times.append(time.perf_counter() - t1)
        looks += b.nnz
        n_cpu += 1
    single = {"value": looks / sum(times), "unit": "lookups/s", "cores": 1,
              "sample": f"{n_cpu} batch(es) of {workload} ({looks} lookups)"}

    # (ii) one unit per table that some field reads
    B = wl.batch
    units = []
    cols = np.concatenate([[0], np.cumsum([wl.tables[f.table].dim for f in wl.fields])])
    for t in range(len(wl.tables)):
        fs = [f for f in range(wl.n_fields) if wl.fields[f].table == t]
        if not fs:
            continue
        sub = copy.copy(wl)
        sub.tables, sub.fields = [wl.tables[t]], [copy.copy(wl.fields[f]) for f in fs]
        for fld in sub.fields:
            fld.table = 0
        units.append((t, fs, SparseOracle(orc, synth, sub)))

    def cut(b, t, fs, su):
        """the unit's share of a batch: its fields' bags, its gradient columns, its distinct rows"""
        ids = np.concatenate([b.ids[b.offsets[f * B]:b.offsets[(f + 1) * B]] for f in fs])
        lens = np.concatenate([np.diff(b.offsets[f * B:(f + 1) * B + 1]) for f in fs])
        offs = np.zeros(len(fs) * B + 1, np.int32)
        offs[1:] = np.cumsum(lens)
        grad = np.ascontiguousarray(np.concatenate([b.grad_out[:, cols[f]:cols[f + 1]] for f in fs], axis=1))
        sb = copy.copy(b)
        sb.ids, sb.offsets, sb.grad_out = np.ascontiguousarray(ids), offs, grad
        key, _ = orc.pack_keys(su.pl, 0, B, sb.ids, sb.offsets)
        uq, _ = orc.unique(key)
        W = synth.table_rows(wl, t, rows=uq.astype(np.int64))
        return sb, [(W, np.zeros(W.shape, np.float32))]

    times2, looks2, n2 = [], 0, 0
    with ThreadPoolExecutor(max_workers=threads) as pool:
        while sum(times2) < budget_s and n2 < 4 * ring:
            b = batches[n2 % ring]
            work = [(su,) + cut(b, t, fs, su) for t, fs, su in units]
            t1 = time.perf_counter()
            list(pool.map(lambda w: w[0].step(w[1], wl.lr, wl.eps, rows=w[2]), work))
            times2.append(time.perf_counter() - t1)
            looks2 += b.nnz
            n2 += 1
    return {"value": looks2 / sum(times2), "unit": "lookups/s", "cores": min(threads, len(units)), "kind": "oracle",
            "host_cores": host_cores,
            "sample": f"{n2} batch(es) of {workload} ({looks2} lookups); the oracle's step functions over "
                      f"{len(units)} independent units (one table and its fields each) on {min(threads, len(units))} "
                      f"threads; rows of the distinct keys and the per-table inputs are staged before the clock starts",
            "single_thread": single}


def main():
    args = parse_args()
    if args.workload:
        print(json.dumps(run_workload(args, args.workload)))
        return
    # default: the 26-field configuration is the headline; the 200-field one, the other configuration the
    # target names, is timed right after it and reported in the same line
    head = run_workload(args, "cfg2")
    import torch
    free, _ = torch.cuda.mem_get_info()
    if free >= 130 * 2**30:
        other = run_workload(args, "cfg3")
        head["workloads"] = {"cfg3": {k: other[k] for k in ("value", "unit", "ms_per_step", "steps", "warmup", "dtype",
                                                           "config", "hbm_model", "roofline", "cpu_baseline",
                                                           "kernels")}}
    else:
        head["workloads"] = {"cfg3": f"skipped: needs about 110 GB of free device memory, {free >> 30} GiB are free"}
    print(json.dumps(head))


if __name__ == "__main__":
    main()
