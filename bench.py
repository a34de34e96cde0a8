#!/usr/bin/env python3
"""Throughput of the Gear Training sparse-part step on one MI355X.

A "step" is one gear_step over one batch of synthetic page views of the "large" workload
(65,536 views, 50M users, 2^25 URL buckets, 4M images with 1024-wide bf16 DFVs, MLP
1152-1024-256-1 on bf16 MFMA, M = 16), inputs resident in HBM.  The full DFV refresh the workload
performs every 500 steps is timed separately and its amortised share is added to ms_per_step.

Prints ONE JSON line: page-views/s, the roofline of the dominant kernel (its duration measured
with HIP events on the launch stream), per-kernel figures, and the CPU oracle timed on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
BYTES = {"f32": 4, "bf16": 2}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--cpu-sample-views", type=int, default=65536,
                    help="views of the oracle's timed sample (0 = skip the CPU baseline)")
    ap.add_argument("--optimizer", choices=["sgd", "adam"], default="sgd",
                    help="sgd is the workload's; adam (beta 0.9 / 0.999, eps 1e-8) is the paper's experiments' choice")
    ap.add_argument("--dense-raw-dim", type=int, default=0,
                    help="close the loop with the stand-in Dense Part (DFV = Wd raw, raw of this width): its backward "
                         "pass takes every step's ready list, its inference pass replaces the periodic refresh")
    ap.add_argument("--expiry", type=int, default=None,
                    help="instead of the periodic full refresh: before every step, recompute (here: replace by "
                         "stand-in rows) the cached DFVs the batch asks for that are at least this many steps old")
    ap.add_argument("--host-counts", action="store_true",
                    help="with --expiry / --dense-raw-dim: read the number of expired rows / of emissions back to the host "
                         "every step instead of leaving it on the device")
    ap.add_argument("--one-stream", action="store_true",
                    help="also run the timed steps with every kernel on one stream, one after another (the per-kernel "
                         "pass always does): the whole command then launches each kernel alone, which is what a "
                         "kernel-trace profile should see when its averages are compared with `kernels`")
    ap.add_argument("--record-mfma", metavar="CSV",
                    help="no GPU work: write profiles/gear_step_large_mfma_busy.txt from the counter CSV of a rocprofv3 --pmc "
                         "SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE run of this benchmark")
    ap.add_argument("--record-traffic", nargs="+", metavar="CSV",
                    help="no GPU work: FETCH_CSV WRITE_CSV [BENCH_LOG]: write profiles/traffic.json and the summary "
                         "profiles/gear_step_large_hbm_traffic.txt from two rocprofv3 --pmc counter CSVs of this benchmark "
                         "(BENCH_LOG: what one of those runs printed, for the algorithmic bytes of the same steps)")
    return ap.parse_args()


class WorkModel:
    """Algorithmic flops / compulsory HBM bytes of each timed launch, from the batch itself."""

    def __init__(self, wl, layers_in, layers_out):
        self.wl, self.lin, self.lout = wl, layers_in, layers_out
        self.counts = np.zeros(wl.n_images, dtype=np.int64)

    def step(self, batch):
        wl = self.wl
        B, nnz, d, D, F = batch.B, batch.nnz, wl.emb_dim, wl.dfv_dim, wl.in_features
        e_emb, e_dfv, e_act = BYTES[wl.emb_dtype], BYTES[wl.dfv_dtype], BYTES[wl.mlp_dtype]
        uu, ul = len(np.unique(batch.user_id)), len(np.unique(batch.url_id))
        img, n_i = np.unique(batch.img_id, return_counts=True)
        p = self.counts[img] % wl.M
        final = (p + n_i) % wl.M
        emits = int(((p + n_i) // wl.M).sum())
        self.counts[img] += n_i
        with_img = int((np.diff(batch.img_off) > 0).sum())
        work = {}
        wgrad_all = 0.0
        for l, (k, n) in enumerate(zip(self.lin, self.lout)):
            if l == len(self.lin) - 1:
                break
            work[f"fwd_gemm_l{l}"] = ("mfma", 2.0 * B * n * k)
            work[f"dgrad_gemm_l{l}"] = ("mfma", 2.0 * B * n * k)
            work[f"wgrad_gemm_l{l}"] = ("mfma", 2.0 * B * n * k)   # one launch per layer (not on this workload)
            wgrad_all += 2.0 * B * n * k
        # dLoss/dx comes from two products: the embedding slots, then the DFV slot
        work["dgrad_gemm_emb"] = ("mfma", 2.0 * B * self.lout[0] * 2 * d)
        work["dgrad_gemm_l0"] = ("mfma", 2.0 * B * self.lout[0] * D)
        work["wgrad_gemm"] = ("mfma", wgrad_all)   # all hidden layers' weight gradients in one launch
        work["gather_pool"] = ("hbm", 12.0 * B + 4.0 * nnz + (uu + ul) * d * e_emb + len(img) * D * e_dfv
                               + B * F * e_act)
        work["embedding_update"] = ("hbm", 16.0 * B + 2.0 * B * d * 4 + 2.0 * (uu + ul) * d * e_emb)
        work["accumulate"] = ("hbm", 40.0 * len(img) + 8.0 * nnz + with_img * D * e_act + int((p != 0).sum()) * D * 4.0
                              + int(((final != 0) | (p != 0)).sum()) * D * 4.0 + emits * D * 4.0)
        return work


CSRC = os.path.join(ROOT, "paper_1806_03925_amd", "csrc")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")
# span -> (parts, source files whose change invalidates the recorded figure); a part is (substring of
# the kernel's name, launches of that kernel in one step, index among them in launch order), and a
# span made of several launches is the sum of its parts
_NS = "gear::(anonymous namespace)::"
TRAFFIC_KERNELS = {
    "gather_pool": ([("k_gather_pool", 1, 0)], ["gather.hip"]),
    "accumulate": ([("k_accumulate", 1, 0)], ["accum.hip"]),
    "embedding_update": ([("k_embedding_chunks", 1, 0), ("k_embedding_spans", 1, 0)], ["update.hip"]),
    "fwd_gemm_l0": ([("k_gemm_nt_dma<0,", 2, 0)], ["gemm.hip"]),
    "fwd_gemm_l1": ([("k_gemm_nt_dma<0,", 2, 1)], ["gemm.hip"]),
    "dgrad_gemm_l1": ([("k_gemm_nt_dma<4,", 1, 0)], ["gemm.hip"]),   # masked by the sign bitmap
    "dgrad_gemm_emb": ([("k_gemm_nt_dma<3, %sNtNarrow>" % _NS, 1, 0)], ["gemm.hip"]),   # the narrow tile shape
    "dgrad_gemm_l0": ([("k_gemm_nt_dma<3, %sNtWide>" % _NS, 1, 0)], ["gemm.hip"]),
    "wgrad_gemm": ([("k_gemm_tn_dma_batch", 1, 0)], ["gemm.hip"]),
}
# launches whose matrix-pipe occupancy is reported (same part notation)
MFMA_KERNELS = {k: v[0] for k, v in TRAFFIC_KERNELS.items() if "gemm" in k}


def source_hash(files):
    h = hashlib.sha256()
    for f in sorted(set(files) | {"gear_internal.hpp"}):
        h.update(open(os.path.join(CSRC, f), "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(span):
    """HBM bytes per launch from the rocprofv3 counter runs, if the kernel's source is unchanged since."""
    if not os.path.exists(TRAFFIC_FILE) or span not in TRAFFIC_KERNELS:
        return None
    rec = json.load(open(TRAFFIC_FILE)).get("kernels", {}).get(span)
    if rec is None or rec.get("source_hash") != source_hash(TRAFFIC_KERNELS[span][1]):
        return None
    return rec["bytes"]


TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "gear_step_large_hbm_traffic.txt")


def write_traffic_summary(rec, refresh_bytes, bench_log=None):
    """The counters of profiles/traffic.json as a table, with the commands that produce them."""
    k, cal = rec["kernels"], rec["calibration"]
    run = "python3 bench.py --steps 3 --warmup 1 --cpu-sample-views 0 --one-stream"
    lines = [
        '# HBM traffic per launch of the timed kernels of gear_step, workload "large" (B=65536), from rocprofv3 counters',
        "# commands (one counter per run; run from the repository root after `cd /tmp && export TMPDIR=/tmp`):",
        f"#   rocprofv3 --pmc FETCH_SIZE -d gpurun_out/pmc_fetch -o f --output-format csv -- {run} > gpurun_out/pmc_fetch.log",
        f"#   rocprofv3 --pmc WRITE_SIZE -d gpurun_out/pmc_write -o w --output-format csv -- {run} > gpurun_out/pmc_write.log",
        "#   python3 bench.py --record-traffic gpurun_out/pmc_fetch/f_counter_collection.csv "
        "gpurun_out/pmc_write/w_counter_collection.csv gpurun_out/pmc_fetch.log",
        f"# calibration: the full DFV refresh (k_refresh) copies {refresh_bytes:,} bytes in and out in the same runs;",
        f"#   FETCH_SIZE reads {refresh_bytes / cal['fetch_bytes_per_count']:.0f} for it -> {cal['fetch_bytes_per_count']:.1f} "
        "bytes per count (the counter's KiB unit sees half of the 128-byte reads)",
        f"#   WRITE_SIZE reads {refresh_bytes / cal['write_bytes_per_count']:.0f} for it -> {cal['write_bytes_per_count']:.1f} "
        "bytes per count",
        f"# averages over the last {k['accumulate']['launches']} launches of a run (its launch-by-launch pass, every kernel alone "
        "on one stream); the machine-readable copy is profiles/traffic.json",
        f"{'launch':16s} {'fetch_MB':>10s} {'write_MB':>10s} {'total_MB':>10s}",
    ]
    for n, v in sorted(k.items(), key=lambda kv: -kv[1]["bytes"]):
        lines.append(f"{n:16s} {v['fetch_bytes'] / 1e6:10.1f} {v['write_bytes'] / 1e6:10.1f} {v['bytes'] / 1e6:10.1f}")
    if bench_log:
        line = [l for l in open(bench_log) if l.startswith("{")][-1]
        alg = {r["name"]: r.get("algorithmic_per_launch") for r in json.loads(line)["kernels"]}
        lines.append("# algorithmic bytes per launch in the same steps (this benchmark's work model): "
                     f"accumulate {alg['accumulate'] / 1e6:.1f} MB, gather_pool {alg['gather_pool'] / 1e6:.1f} MB, "
                     f"embedding_update {alg['embedding_update'] / 1e6:.1f} MB")
        lines.append("# (accumulate's grows with the step number, as more images carry a partial sum that has to be read: "
                     "530 MB in the first step after initialisation, 720 MB in the eighth, about 850 MB around step 100)")
    lines += ["# the excess is re-reads of dLoss/dx rows (accumulate: one row per occurrence, 4.5 per view) and of cached "
              "DFV rows (gather) that miss in L2.",
              "# dgrad_gemm_l1 reads the 8 MB sign bitmap of the first hidden layer instead of its 134 MB of activations."]
    open(TRAFFIC_SUMMARY, "w").write("\n".join(lines) + "\n")


def record_traffic(fetch_csv, write_csv, bench_log=None, refresh_bytes=0):
    """Turn two `rocprofv3 --pmc` runs of this benchmark (FETCH_SIZE, then WRITE_SIZE; counter CSVs) into
    profiles/traffic.json.  Each counter is scaled by what it reads for the full DFV refresh, a plain
    copy of `refresh_bytes` in and out."""
    import csv

    def per_kernel(path, counter):
        rows = [r for r in csv.DictReader(open(path)) if r["Counter_Name"] == counter]
        rows.sort(key=lambda r: int(r["Dispatch_Id"]))
        by_name = {}
        for r in rows:
            by_name.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
        return by_name

    def pick(by_name, sub):
        hits = [v for k, v in by_name.items() if sub in k]
        assert len(hits) == 1, (sub, [k for k in by_name if sub in k])
        return hits[0]

    out = {"unit": "bytes per launch", "calibration": {}, "kernels": {}}
    # with the run's own line at hand: only the launches of its last pass (the `steps` steps that are timed launch
    # by launch and whose algorithmic bytes the line carries), so that both figures are of the same steps
    last = None
    if bench_log:
        last = int(json.loads([l for l in open(bench_log) if l.startswith("{")][-1])["steps"])
    tables = {}
    for key, path, counter in (("fetch", fetch_csv, "FETCH_SIZE"), ("write", write_csv, "WRITE_SIZE")):
        tables[key] = per_kernel(path, counter)
        copy = pick(tables[key], "k_refresh")
        # the first launch of that kernel is the full refresh; the later ones (the random-row probe) are smaller
        assert len(copy) >= 1 and copy[0] == max(copy)
        out["calibration"][key + "_bytes_per_count"] = refresh_bytes / copy[0]
    for span, (parts, files) in TRAFFIC_KERNELS.items():
        rec = {"source_hash": source_hash(files)}
        for key in ("fetch", "write"):
            rec[key + "_bytes"] = 0.0
            for sub, per_step, index in parts:
                vals = pick(tables[key], sub)
                assert len(vals) % per_step == 0, (span, len(vals))
                mine = vals[index::per_step]
                if last:
                    mine = mine[-last:]
                rec[key + "_bytes"] += float(np.mean(mine)) * out["calibration"][key + "_bytes_per_count"]
                rec["launches"] = len(mine)
        rec["bytes"] = rec["fetch_bytes"] + rec["write_bytes"]
        out["kernels"][span] = rec
    json.dump(out, open(TRAFFIC_FILE, "w"), indent=1, sort_keys=True)
    write_traffic_summary(out, refresh_bytes, bench_log)
    print(json.dumps(out, indent=1, sort_keys=True))


MFMA_SUMMARY = os.path.join(ROOT, "profiles", "gear_step_large_mfma_busy.txt")


def record_mfma(counter_csv, n_cus=256, n_xcds=8):
    """Matrix-pipe occupancy of the MLP's products from one `rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES
    GRBM_GUI_ACTIVE` run of this benchmark: busy cycles summed over all SIMDs, divided by the cycles the
    kernel was on the device (the counter adds up the XCDs' cycle counts) times the number of SIMDs."""
    import csv
    rows = sorted(csv.DictReader(open(counter_csv)), key=lambda r: int(r["Dispatch_Id"]))
    by = {}
    for r in rows:
        by.setdefault((r["Kernel_Name"], r["Counter_Name"]), []).append(float(r["Counter_Value"]))

    def pick(sub, counter):
        hits = [v for (k, c), v in by.items() if sub in k and c == counter]
        assert len(hits) == 1, (sub, counter)
        return hits[0]

    run = "python3 bench.py --steps 3 --warmup 1 --cpu-sample-views 0 --one-stream"
    lines = ['# Matrix-pipe (MFMA) occupancy of the MLP products of gear_step, workload "large" (B=65536), every kernel alone',
             "# command (from the repository root after `cd /tmp && export TMPDIR=/tmp`):",
             f"#   rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE -d gpurun_out/pmc_mfma -o m --output-format csv -- {run}",
             "#   python3 bench.py --record-mfma gpurun_out/pmc_mfma/m_counter_collection.csv",
             f"# busy = SQ_VALU_MFMA_BUSY_CYCLES (summed over the {n_cus * 4} SIMDs); active = GRBM_GUI_ACTIVE / {n_xcds} (the counter",
             f"# adds up the {n_xcds} XCDs); occupancy = busy / (active * {n_cus * 4}).  One bf16 32x32x16 MFMA keeps a pipe busy 32 cycles,",
             "# so busy / 32 * 32768 flop is the product's flop count (checked in the last column).",
             f"{'launch':16s} {'launches':>8s} {'busy_cycles':>14s} {'active_cycles':>14s} {'occupancy':>10s} {'GFLOP_from_busy':>16s}"]
    for span, parts in MFMA_KERNELS.items():
        busy = act = 0.0
        n = 0
        for sub, per_step, index in parts:
            b, a = pick(sub, "SQ_VALU_MFMA_BUSY_CYCLES")[index::per_step], pick(sub, "GRBM_GUI_ACTIVE")[index::per_step]
            busy, act, n = busy + float(np.mean(b)), act + float(np.mean(a)) / n_xcds, len(b)
        lines.append(f"{span:16s} {n:8d} {busy:14.0f} {act:14.0f} {busy / (act * n_cus * 4):10.3f} {busy / 32 * 32768 / 1e9:16.1f}")
    open(MFMA_SUMMARY, "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))


def cpu_baseline(wl, views):
    """The oracle as it stands, timed on this host over one batch of `views` page views: once with its
    matrix products on one thread, once with the BLAS thread pool as found (everything else in the
    oracle is a plain Python loop on one thread either way)."""
    from threadpoolctl import threadpool_info, threadpool_limits

    from gear_inputs import PageViewSource
    from oracle.from_workload import oracle_for
    batch = PageViewSource(wl).batch(0, batch=views)

    def timed(limit):
        orc = oracle_for(wl)
        orc.user_emb.prefetch(batch.user_id)
        orc.url_emb.prefetch(batch.url_id)
        orc.dfv.prefetch(batch.img_id)
        with threadpool_limits(limits=limit):
            t0 = time.perf_counter()
            orc.step(batch, float(np.float32(wl.lr)))
            return time.perf_counter() - t0

    dt1 = timed(1)
    dtn = timed(None)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    what = (f"1 oracle step over one batch of {views} views drawn the way the {wl.name} workload draws its batches "
            "(table rows materialised beforehand)")
    return {"value": views / dt1, "unit": "page-views/s", "cores": 1, "threads": 1, "kind": "oracle",
            "sample": f"{what}, matrix products limited to one thread: {dt1:.1f} s",
            "all_threads": {"value": views / dtn, "unit": "page-views/s", "cores": int(threads), "threads": int(threads),
                            "sample": f"the same step with the BLAS thread pool as found ({threads} threads for the "
                                      f"matrix products, the rest of the oracle on one): {dtn:.1f} s"}}


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this library runs on one GPU only (got --gpus {args.gpus}); "
              "the step has no multi-GPU path", file=sys.stderr)
        sys.exit(2)

    from gear_inputs import PageViewSource, get_workload

    wl = get_workload(args.workload)
    if args.record_mfma:
        record_mfma(args.record_mfma)
        return
    if args.record_traffic:
        if len(args.record_traffic) not in (2, 3):
            sys.exit("--record-traffic takes FETCH_CSV WRITE_CSV [BENCH_LOG]")
        record_traffic(*args.record_traffic, refresh_bytes=wl.n_images * wl.dfv_dim * BYTES[wl.dfv_dtype])
        return

    import torch

    import paper_1806_03925_amd as g

    torch.cuda.set_device(0)
    cfg = g.config_for(wl)
    st = g.GearState(cfg)
    g.gear_init_tables(st)
    g.gear_fill_normal(st.dfv_cache, wl.n_images, wl.dfv_dim, wl.seed, 3, wl.dfv_std)
    torch.cuda.synchronize()

    K, W = args.steps, args.warmup
    src = PageViewSource(wl)
    # a batch of its own for every step (warm-up, timed, spread, waited, launch by launch), up to 160 (320 MB on the device)
    pool = min(W + 3 * K + min(K, 10), 160)
    host = [src.batch(i) for i in range(pool)]
    dev = [g.DeviceBatch.from_host(b) for b in host]
    lr = float(wl.lr)
    lin = [wl.in_features] + list(wl.layers[:-1])
    model = WorkModel(wl, lin, list(wl.layers))

    # expiry mode (Section 4.1, Table 2): the rows a batch asks for are recomputed when they are
    # `expiry` steps old.  The Dense Part that would recompute them is not part of this library; a
    # pool of random rows stands in for its output, so what is timed is finding the expired rows,
    # writing and stamping them, and the step.
    expiry = args.expiry
    refreshed = []
    if expiry is not None:
        stamp = torch.zeros(wl.n_images, dtype=torch.int32, device="cuda")
        fresh_pool = torch.empty((wl.max_nnz, wl.dfv_dim), dtype=st.dfv_cache.dtype, device="cuda")
        g.gear_fill_normal(fresh_pool, wl.max_nnz, wl.dfv_dim, wl.seed + 2, 3, wl.dfv_std)

    def one_step(i):
        if expiry is not None:
            ids, n_dev = g.gear_expired_ids(st, dev[i % pool].img_id, stamp, i, expiry)
            if args.host_counts:
                n = int(n_dev.item())                  # a caller that has to know how many rows to recompute
                refreshed.append(n)
                if n:
                    g.gear_refresh_dfv(st, ids[:n], fresh_pool[:n])
                    g.gear_stamp_dfv(st, stamp, ids[:n], i)
            else:                                      # the count stays on the device, the host runs ahead
                refreshed.append(n_dev)
                g.gear_refresh_dfv_n(st, ids, fresh_pool, n_dev)
                g.gear_stamp_dfv_n(st, stamp, ids, n_dev, i)
        if adam is None:
            g.gear_step(st, dev[i % pool], wl.M, lr)
        else:
            g.gear_step_adam(st, dev[i % pool], wl.M, lr, adam)
        if dense is not None:
            if args.host_counts:
                n_ready = int(st.n_ready.item())       # a caller that has to know how many arrived
                dense.backward(st.ready_ids, st.ready_grads, n_ready, lr)
            else:
                dense.backward_n(st.ready_ids, st.ready_grads, st.n_ready, lr)

    adam = g.AdamMoments(st) if args.optimizer == "adam" else None
    dense, dense_rows = None, 1 << 18
    if args.dense_raw_dim:
        R = args.dense_raw_dim
        raw = torch.empty((wl.n_images, R), dtype=torch.float32, device="cuda")
        wd = torch.empty((wl.dfv_dim, R), dtype=torch.float32, device="cuda")
        g.gear_fill_normal(raw, wl.n_images, R, wl.seed + 3, 3, 1.0)
        g.gear_fill_normal(wd, wl.dfv_dim, R, wl.seed + 4, 3, R ** -0.5)
        dense = g.DenseStandIn(st, raw, wd, max_rows=max(dense_rows, wl.max_nnz))
    st.one_stream = args.one_stream
    it = 0
    for _ in range(W):
        one_step(it)
        model.step(host[it % pool])
        it += 1
    torch.cuda.synchronize()
    refreshed.clear()
    t0 = time.perf_counter()
    for i in range(K):
        one_step(it)
        it += 1
    torch.cuda.synchronize()
    loop_ms = (time.perf_counter() - t0) * 1e3
    for i in range(it - K, it):
        model.step(host[i % pool])
    assert int(st.status.item()) == 0 and np.isfinite(float(st.loss.item()))
    loss = float(st.loss.item())
    refreshed_per_step = float(np.mean([int(r) for r in refreshed])) if refreshed else None   # device words are read here

    # spread of the step time: the same again with an event between steps (each costs the launch
    # stream a few microseconds, which is why the timed steps above carry none)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    marks[0].record()
    for i in range(K):
        one_step(it)
        marks[i + 1].record()
        it += 1
    torch.cuda.synchronize()
    step_ms = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(K)])
    for i in range(it - K, it):
        model.step(host[i % pool])

    # a caller that waits for every step before it issues the next (the host is never ahead of the
    # device): host wall clock from the call to the end of the wait
    n_waited = min(K, 10)
    waited = []
    for i in range(n_waited):
        torch.cuda.synchronize()
        t_call = time.perf_counter()
        one_step(it)
        torch.cuda.synchronize()
        waited.append((time.perf_counter() - t_call) * 1e3)
        it += 1
    for i in range(it - n_waited, it):
        model.step(host[i % pool])

    # per-kernel durations: the same steps again with HIP events around every launch, all on one
    # stream, so that a duration is that of the kernel alone (in the timed steps above, parts of a
    # step run side by side on two streams and share the device)
    st.profile = g.GearProfile()
    st.one_stream = True
    spans, work = {}, {}
    for _ in range(K):
        one_step(it)
        torch.cuda.synchronize()
        for name, ms in st.profile.spans():
            spans.setdefault(name, []).append(ms)
        for name, (bound, amount) in model.step(host[it % pool]).items():
            work.setdefault(name, [bound, 0.0])[1] += amount / K
        it += 1
    st.profile.close()
    st.profile = None
    st.one_stream = args.one_stream

    # the workload's periodic full DFV refresh (new vectors stand in for a Dense-Part inference pass)
    refresh_ms, copy_gbs, dense_refresh_ms, row_copy_gbs = 0.0, None, None, None
    refresh_every = 0 if expiry is not None else wl.refresh_every   # expiry mode replaces the periodic full refresh
    if wl.refresh_every:
        fresh = torch.empty_like(st.dfv_cache)
        g.gear_fill_normal(fresh, wl.n_images, wl.dfv_dim, wl.seed + 1, 3, wl.dfv_std)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        g.gear_refresh_dfv(st, None, fresh)
        e1.record()
        if dense is not None:
            # the refresh as the closed loop does it: inference for the whole image set, a slab at a time
            d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            d0.record()
            for c0 in range(0, wl.n_images, dense_rows):
                ids = torch.arange(c0, min(wl.n_images, c0 + dense_rows), dtype=torch.int32, device="cuda")
                g.gear_refresh_dfv(st, ids, dense.infer(ids))
            d1.record()
            torch.cuda.synchronize()
            dense_refresh_ms = d0.elapsed_time(d1)
        torch.cuda.synchronize()
        refresh_ms = e0.elapsed_time(e1)
        # the refresh is a plain copy of the whole cache: what this device's HBM sustains in practice
        copy_gbs = 2.0 * wl.n_images * wl.dfv_dim * BYTES[wl.dfv_dtype] / (refresh_ms * 1e-3) / 1e9
        # ... and the same kernel over as many distinct random rows as a batch has occurrences: what moving whole
        # rows with no reuse can reach (rows read in order from the fresh table, written to random rows of the cache)
        n_rows = min(wl.max_nnz // 2, wl.n_images // 2)
        ids = torch.randperm(wl.n_images, device="cuda")[:n_rows].to(torch.int32)
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        rows = fresh[:n_rows]                                # the call takes its row count from this argument
        g.gear_refresh_dfv(st, ids, rows)                    # once untimed
        torch.cuda.synchronize()
        r0.record()
        for _ in range(5):
            g.gear_refresh_dfv(st, ids, rows)
        r1.record()
        torch.cuda.synchronize()
        row_copy_gbs = 2.0 * n_rows * wl.dfv_dim * BYTES[wl.dfv_dtype] / (r0.elapsed_time(r1) / 5 * 1e-3) / 1e9
        del fresh, rows

    per_refresh = dense_refresh_ms if dense_refresh_ms is not None else refresh_ms
    ms_per_step = loop_ms / K + (per_refresh / refresh_every if refresh_every else 0.0)
    value = wl.batch / (ms_per_step * 1e-3)

    kernels = []
    for name, samples in spans.items():
        launches = len(samples) / K
        avg_ms = float(np.mean(samples))
        row = {"name": name, "ms_per_step": avg_ms * launches, "launches_per_step": launches}
        if name in work:
            bound, amount = work[name]
            if bound == "mfma":
                row.update(bound="mfma", achieved=amount / (avg_ms * 1e-3) / 1e12, unit="TFLOP/s",
                           peak=MFMA_PEAK_TFLOPS[wl.mlp_dtype])
            else:
                row.update(bound="hbm", achieved=amount / (avg_ms * 1e-3) / 1e9, unit="GB/s", peak=HBM_PEAK_GBS)
                if copy_gbs:
                    row["frac_of_measured_copy"] = row["achieved"] / copy_gbs
            row["frac"] = row["achieved"] / row["peak"]
            row["algorithmic_per_launch"] = amount
            row["traffic"] = recorded_traffic(name)
        kernels.append(row)
    kernels.sort(key=lambda r: -r["ms_per_step"])
    dominant = next(r for r in kernels if "bound" in r)
    roofline = {"kernel": dominant["name"], "bound": dominant["bound"], "achieved": dominant["achieved"],
                "peak": dominant["peak"], "unit": dominant["unit"], "frac": dominant["frac"],
                "avg_launch_ms": dominant["ms_per_step"] / dominant["launches_per_step"],
                "traffic": recorded_traffic(dominant["name"]),
                "measured": "kernel alone: per-launch HIP events, all launches on one stream"}

    out = {
        "metric": "page-views/sec per gear_step at 1 GPU", "value": value, "unit": "page-views/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": wl.mlp_dtype, "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "n_users": wl.n_users, "n_urls": wl.n_urls,
                   "n_images": wl.n_images, "emb_dim": wl.emb_dim, "dfv_dim": wl.dfv_dim,
                   "mlp": [wl.in_features, *wl.layers], "M": wl.M, "zipf_s": wl.zipf_image,
                   "refresh_every": refresh_every, "refresh_ms": refresh_ms, "expiry_steps": expiry, "optimizer": args.optimizer,
                   "dense_raw_dim": args.dense_raw_dim or None, "dense_refresh_ms": dense_refresh_ms,
                   "expired_rows_per_step": refreshed_per_step,
                   "loop_ms_per_step": loop_ms / K, "profiled_ms_per_step": sum(r["ms_per_step"] for r in kernels),
                   "step_ms_p10_p50_p90": [float(np.percentile(step_ms, q)) for q in (10, 50, 90)],
                   "waited_step_ms_median": float(np.median(waited)),
                   "hbm_copy_GBs": copy_gbs, "hbm_random_row_copy_GBs": row_copy_gbs,
                   "timed_steps_on_one_stream": bool(args.one_stream)},
        "loss": loss,
        "roofline": roofline,
        "kernels": kernels,
    }
    if args.cpu_sample_views > 0:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample_views)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
