#!/usr/bin/env python3
"""Benchmark of the dynamic-GNN hot path on one MI355X.

A step is one forward pass over one GPU's block of snapshots of a seeded synthetic dynamic graph:
for every snapshot after the first, rebuild its CSR on the GPU from the previous snapshot and the
graph difference (c5: lists copied from pinned host memory on a second stream inside the timed region;
the other workloads: lists resident in HBM), then H = X W and Z = relu(A~ H) per GCN layer;
workloads with a window finish with the M-transform over the block.  Throughput is the paper's
definition (Section "Scaling Study", weak scaling): edges summed over the processed snapshots
divided by time.

Prints ONE JSON line.  Besides the throughput it carries
  roofline      for the stage that takes the most time: algorithmic bytes per call / its average
                duration, measured here with event pairs on the launch stream, against 8 TB/s;
  cpu_baseline  the CPU oracle (oracle/) timed on the host cores on a bounded sample.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def progress(msg):
    """One line per finished step on stderr, so that a long run is never silent."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--settle-seconds", type=float, default=1.5,
                    help="untimed passes of the same step before the warm-up steps, for this long: the device reaches its "
                         "steady clocks and the pinned buffers have been read once (with 2 warm-up steps alone the timed "
                         "steps of c5 come out 6 %% slower than after 20)")
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--n", type=int, default=0, help="run the workload's recipe at another vertex count (debugging)")
    ap.add_argument("--T", type=int, default=0, help="override the number of snapshots (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="stop the oracle sample after this much work")
    ap.add_argument("--pinned", action="store_true",
                    help="difference lists in pinned host memory, copied on a second stream inside the timed region "
                         "(the default for c5, whose definition says so)")
    ap.add_argument("--resident", action="store_true", help="difference lists already in HBM (the default except for c5)")
    ap.add_argument("--no-train", action="store_true", help="skip the training-step (forward + backward) measurement")
    ap.add_argument("--graph", action="store_true",
                    help="also time the forward pass replayed as one HIP graph (for launch-bound small workloads)")
    ap.add_argument("--cdgcn", action="store_true",
                    help="also time the forward pass of one CD-GCN layer (skip-concat GCN + LSTM over time) over the block")
    ap.add_argument("--weighted", action="store_true",
                    help="also time one step of the path for snapshots that carry a value per entry")
    ap.add_argument("--smoothing", action="store_true",
                    help="also time the sliding-window sum of the block's snapshots (edge life 4) computed on the device")
    ap.add_argument("--smoothing-sum-only", action="store_true",
                    help="with --smoothing: only the series of sliding-window sums and the normalisation (no smoothed pass, no training step)")
    ap.add_argument("--two-streams", action="store_true",
                    help="also time the step with the next snapshot's rebuild and X W on a second stream beside the aggregation")
    ap.add_argument("--working-sets", action="store_true",
                    help="also time the aggregation with its gathers confined to working sets of known size")
    ap.add_argument("--mproduct-band", action="store_true",
                    help="also time the M-transform with explicit coefficients and window 32")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline figure (and whatever is asked for explicitly): skip the CD-GCN, weighted and smoothing figures")
    ap.add_argument("--gen-device", default="cuda", choices=["cuda", "cpu"],
                    help="where the seeded generator runs; cpu keeps every dispatch of a profiled run the library's own")
    ap.add_argument("--repeat-features", action="store_true",
                    help="X_t = X_1 for every t (counter runs: the traffic does not depend on the values)")
    ap.add_argument("--natural-labels", action="store_true",
                    help="R-MAT workloads: keep the generator's vertex labels (locality) instead of scrambling them")
    return ap.parse_args()


def algorithmic_bytes(blk, stage, t=None):
    """Bytes the method itself must move per call of a stage (index = 4 B, no value array)."""
    s = blk.x[0].element_size()
    n, f = blk.n, blk.f
    if stage == "delta_rebuild":
        n_delta = blk.deltas[t - 2][0].numel() + blk.deltas[t - 2][2].numel()
        return 4 * blk.nnz[t - 2] + 4 * blk.nnz[t - 1] + 16 * n + 16 * n_delta
    if stage == "feature_transform":
        return 2 * s * n * f + s * f * f
    if stage == "spmm":            # lower bound: every row of H fetched once
        return 4 * blk.nnz[t - 1] + 8 * n + 2 * s * n * f
    if stage in ("mproduct", "mproduct_backward"):
        return 2 * s * n * f * blk.T
    if stage == "spmm_transposed":
        return 4 * blk.nnz[t - 1] + 8 * n + 2 * s * n * f
    if stage == "relu_backward":   # gradient in, activation in, masked gradient out
        return 3 * s * n * f + 4 * n
    if stage in ("weight_grad", "input_grad"):
        return 2 * s * n * f + s * f * f
    raise KeyError(stage)


STAGE_SOURCES = {"spmm": ("spmm.hip", "common.hpp"), "delta_rebuild": ("delta_rebuild.hip", "common.hpp"),
                 "feature_transform": ("feature_transform.hip", "common.hpp"), "mproduct": ("mproduct.hip", "common.hpp")}


def kernel_source_digest(stage):
    """sha256 over the source files a stage's kernels are compiled from (what a committed counter profile is tied to)."""
    import hashlib
    h = hashlib.sha256()
    for name in STAGE_SOURCES[stage]:
        with open(os.path.join(ROOT, "paper_2109_07893_amd", "csrc", name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def committed_traffic(workload, stage):
    """(bytes per call, where they come from).  The bytes are rocprofv3 FETCH_SIZE + WRITE_SIZE of the stage's kernels
    from the committed counter summary, which names the digest of the kernel sources it was taken on; a summary taken
    on other sources is refused (None), so the figure cannot go stale silently."""
    rel = os.path.join("profiles", f"{stage}_{workload}_hbm_traffic.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, "no committed counter summary for this stage and workload"
    text = open(path).read()
    m = re.search(r"^traffic_bytes_per_call:\s*([0-9.eE+]+)", text, flags=re.M)
    d = re.search(r"^kernel_source_digest:\s*([0-9a-f]+)", text, flags=re.M)
    if not m:
        return None, f"{rel} holds no traffic_bytes_per_call line"
    now = kernel_source_digest(stage)
    if not d or d.group(1) != now:
        return None, (f"{rel} was taken on kernel sources {d.group(1) if d else '(not recorded)'}, the build now has {now}: "
                      "refused, retake the counter passes")
    return float(m.group(1)), f"{rel} (separate rocprofv3 --pmc passes on kernel sources {now})"


def cpu_baseline(wl, blk, first, budget_s):
    """The oracle as it stands on the host cores, over the first timesteps of the same block: one thread first (the
    baseline figure), then all threads the box gives it."""
    import numpy as np
    import oracle
    n = blk.n
    ws = [w.detach().cpu().double().numpy() for w in blk.w]
    all_threads = oracle.num_threads()

    def run(threads, t_stop, budget):
        oracle.set_threads(threads)
        rp = blk.rowptr1.cpu().numpy()
        ci = blk.colidx1.cpu().numpy()
        edges, spent, done = 0, 0.0, []
        for t in range(1, min(blk.T, t_stop) + 1):
            lists = [x.cpu().numpy() for x in blk.deltas[t - 2]] if t >= 2 else None
            x = blk.x[t - 1].detach().cpu().double().numpy()
            t0 = time.perf_counter()
            if t >= 2:
                rp, ci = oracle.delta_apply(n, rp, ci, *lists)
            if t >= first:
                val = oracle.gcn_values(rp, ci)
                cur = x
                for w in ws:
                    cur = oracle.spmm(rp, ci, oracle.xw(cur, w), relu=True, val=val)
            dt = time.perf_counter() - t0
            if t >= first:
                spent += dt
                edges += int(ci.size)
                done.append(t)
            if spent >= budget:
                break
        progress(f"oracle with {threads} thread(s): t={done[0]}..{done[-1]} in {spent:.1f} s")
        return {"value": edges / spent if spent > 0 else None, "unit": "edges/s", "cores": threads, "seconds": round(spent, 3),
                "sample": f"timesteps t={done[0]}..{done[-1]} of the same block (rebuild + {len(ws)} GCN layer(s), "
                          f"no M-transform), full graph, {edges} edges"}

    try:
        model = next(l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name"))
    except (OSError, StopIteration):
        model = "unknown"
    # one thread: a single timed timestep of a large workload is already tens of seconds; all threads: at least three
    single = run(1, first + 2, budget_s)
    multi = run(all_threads, first + 2, 3 * budget_s)
    oracle.set_threads(all_threads)
    out = dict(single)
    out.update({"kind": "oracle", "all_cores": multi, "nproc": os.cpu_count(), "cpu_model": model})
    return out


def gather_working_sets(args, wl, blk, dev):
    """dgnn_spmm on the first snapshot's row structure with the column indices replaced, so that the gathered rows of H
    come from working sets of known size: inside one L2 (1 MB), inside the Infinity Cache (32 and 128 MB), beyond it
    (512 MB), or spread uniformly over the whole of H.  Tells what bounds the aggregation on the real columns: an extra figure."""
    import torch
    import paper_2109_07893_amd as dg
    n, f, nnz = blk.n, blk.f, blk.nnz[0]
    h = blk.x[0]
    z = torch.empty_like(h)
    dinv = torch.empty(n, dtype=torch.float32, device=dev)
    dg.csr_dinv(blk.rowptr1, dinv)
    ws = torch.empty(dg.spmm_workspace(n, nnz, f), dtype=torch.uint8, device=dev)
    row_bytes = f * h.element_size()
    patterns = [("the workload's columns", blk.colidx1)]
    gen = torch.Generator(device=dev).manual_seed(wl.seed)
    # uniformly random inside the working set: every wavefront, and so every L2, sees all of it (columns that follow
    # the entry index would hand each L2 a share of its own)
    for size in (1 << 20, 32 << 20, 128 << 20, 512 << 20):
        m = max(1, min(n, size // row_bytes))
        patterns.append((f"columns inside {size >> 20} MB of H", torch.randint(0, m, (nnz,), generator=gen, device=dev, dtype=torch.int32)))
    patterns.append((f"uniformly random columns ({n * row_bytes / 1e9:.2f} GB of H)", torch.randint(0, n, (nnz,), generator=gen, device=dev, dtype=torch.int32)))
    out = {"entries": nnz, "gathered_bytes": nnz * row_bytes, "cases": []}
    for label, cols in patterns:
        for _ in range(2):
            dg.spmm(blk.rowptr1, cols, nnz, dinv, h, z, ws, flags=dg.DGNN_RELU | dg.DGNN_H_PRESCALED)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            dg.spmm(blk.rowptr1, cols, nnz, dinv, h, z, ws, flags=dg.DGNN_RELU | dg.DGNN_H_PRESCALED)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        out["cases"].append({"columns": label, "avg_ms": round(ms, 4), "gather_GBps": round(nnz * row_bytes / (ms * 1e-3) / 1e9, 1)})
    return out


def mproduct_band(args, wl, blk, dev):
    """The M-transform with explicit coefficients and the longest window (32) over frames of the workload's shape:
    an extra figure for the kernel that keeps its ring as raw pieces."""
    import torch
    import paper_2109_07893_amd as dg
    n, f, T, w = blk.n, blk.f, 40, 32
    free, _ = torch.cuda.mem_get_info(dev)
    frame = n * f * blk.x[0].element_size()
    T = int(max(w + 1, min(T, 0.4 * free // frame)))
    z = torch.empty((T, n, f), dtype=blk.x[0].dtype, device=dev).normal_()
    band = torch.full((T, w), 1.0 / w, device=dev)
    for _ in range(2):
        dg.mproduct(z, z, w, m_band=band)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        dg.mproduct(z, z, w, m_band=band)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    return {"window": w, "frames": T, "avg_ms": round(ms, 3), "algorithmic_GBps": round(2 * T * frame / (ms * 1e-3) / 1e9, 1)}


def weighted_step(args, wl, blk, dev):
    """A_2 from A_1 with a value per stored entry (values carried, added entries bring theirs, 5 % of the
    survivors get a new one), then Z = relu(V H) on the rebuilt snapshot: an extra figure."""
    import torch
    import paper_2109_07893_amd as dg
    n, f = blk.n, blk.f
    gen = torch.Generator(device=dev).manual_seed(wl.seed)
    nnz1 = blk.nnz[0]
    ar, ac, dr, dc = blk.deltas[0]
    val1 = torch.rand(nnz1, generator=gen, device=dev) + 0.5
    add_val = torch.rand(ar.numel(), generator=gen, device=dev) + 0.5
    # update list: a seeded 5 % of A_1's entries that are not deleted
    pos = torch.randint(0, nnz1, (nnz1 // 20,), generator=gen, device=dev).unique()
    rows = torch.searchsorted(blk.rowptr1.to(torch.int64), pos, right=True) - 1
    keys = (rows << 32) | blk.colidx1[pos].to(torch.int64)
    keys = keys[~torch.isin(keys, (dr.to(torch.int64) << 32) | dc.to(torch.int64))]
    ur, uc = (keys >> 32).to(torch.int32), (keys & 0xffffffff).to(torch.int32)
    uv = torch.rand(ur.numel(), generator=gen, device=dev) + 2.0
    cap = blk.nnz[1]
    rpn = torch.empty(n + 1, dtype=torch.int32, device=dev)
    cin = torch.empty(cap, dtype=torch.int32, device=dev)
    vn = torch.empty(cap, dtype=torch.float32, device=dev)
    ws_r = torch.empty(dg.delta_rebuild_workspace(n, nnz1, ar.numel(), dr.numel()), dtype=torch.uint8, device=dev)
    ws_s = torch.empty(dg.spmm_workspace(n, cap, f), dtype=torch.uint8, device=dev)
    h, z = blk.x[1], torch.empty_like(blk.x[1])

    def rebuild():      # the update list is sorted by (row, col): the merge consumes it
        dg.delta_rebuild_weighted(blk.rowptr1, blk.colidx1, val1, nnz1, (ar, ac, add_val), (dr, dc), (ur, uc, uv), rpn, cin,
                                  vn, ws_r, flags=dg.DGNN_UPDATES_SORTED)

    def rebuild_any_order():      # the same list handed over as unordered: a pass of its own after the merge
        dg.delta_rebuild_weighted(blk.rowptr1, blk.colidx1, val1, nnz1, (ar, ac, add_val), (dr, dc), (ur, uc, uv), rpn, cin,
                                  vn, ws_r)

    def aggregate():
        dg.spmm_weighted(rpn, cin, vn, cap, h, z, ws_s, flags=dg.DGNN_RELU)

    dinv_w = torch.empty(n, dtype=torch.float32, device=dev)
    ws_d = torch.empty(dg.csr_weighted_dinv_workspace(cap), dtype=torch.uint8, device=dev)

    def normalise():
        dg.csr_weighted_dinv(rpn, vn, cap, dinv_w, ws_d)

    out = {}
    s = h.element_size()
    rebuild_bytes = 8 * nnz1 + 8 * cap + 16 * n + 20 * (ar.numel() + dr.numel()) + 12 * ur.numel()
    for name, fn, byts in (("delta_rebuild_weighted", rebuild, rebuild_bytes),
                           ("delta_rebuild_weighted_updates_in_any_order", rebuild_any_order, rebuild_bytes),
                           ("spmm_weighted", aggregate, 8 * cap + 4 * n + 2 * s * n * f),
                           ("csr_weighted_dinv", normalise, 4 * cap + 8 * n)):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        out[name] = {"avg_ms": round(ms, 4), "algorithmic_bytes_per_call": int(byts),
                     "algorithmic_GBps": round(byts / (ms * 1e-3) / 1e9, 1)}
    out["lists"] = {"added": int(ar.numel()), "deleted": int(dr.numel()), "value_updates": int(ur.numel())}
    return out


def two_stream_steps(args, wl, blk, dev):
    """The timed step once more with the rebuild and X W of snapshot t+1 on a second stream while snapshot t is
    aggregated (BlockRunner's overlap mode), beside the same step on one stream: an extra figure, the headline keeps
    the one-stream pass that the per-stage figures and the profiles describe."""
    import torch
    from paper_2109_07893_amd.pipeline import BlockRunner
    runner = BlockRunner(blk)
    runner.load_first()
    first = 1 if blk.window else 2
    edges = sum(blk.nnz[first - 1:])

    def timed(fn, finish=None):
        for _ in range(max(args.warmup, 1)):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        el = (time.perf_counter() - t0) / args.steps
        if finish:
            finish()
            torch.cuda.synchronize()
        return {"ms_per_step": round(el * 1e3, 3), "value": edges / el, "unit": "edges/s"}

    out = {"lists_resident": {"one_stream": timed(lambda: runner.run_resident(first=first)),
                              "two_streams": timed(lambda: runner.run_resident(first=first, overlap=True))}}
    if blk.pinned is not None:
        out["lists_from_pinned_host"] = {
            "one_stream": timed(lambda: runner.run_from_pinned(first=first, prefetch_next=True),
                                lambda: runner.run_from_pinned(first=first)),
            "two_streams": timed(lambda: runner.run_from_pinned(first=first, prefetch_next=True, overlap=True),
                                 lambda: runner.run_from_pinned(first=first, overlap=True))}
    out["note"] = ("two_streams: rebuild of A_t+1 and X_t+1 W enqueued on a second stream, at most one snapshot ahead of the "
                   "aggregations; same kernels, same operands, bit-identical results; one more H buffer")
    return out


def smoothing_steps(args, wl, blk, dev, life=4):
    """S_t = S_{t-1} + A_t - A_{t-life} over the block with all raw snapshots resident (rebuilt on the device from
    the difference lists), then the normalisation of the last S_t: an extra figure."""
    import torch
    import paper_2109_07893_amd as dg
    n = blk.n
    snaps = [(blk.rowptr1, blk.colidx1, blk.nnz[0])]
    ws_r = torch.empty(dg.delta_rebuild_workspace(n, max(blk.nnz), max(int(d[0].numel()) for d in blk.deltas),
                                                  max(int(d[2].numel()) for d in blk.deltas)), dtype=torch.uint8, device=dev)
    for t in range(2, blk.T + 1):
        ar, ac, dr, dc = blk.deltas[t - 2]
        rp = torch.empty(n + 1, dtype=torch.int32, device=dev)
        ci = torch.empty(blk.nnz[t - 1], dtype=torch.int32, device=dev)
        dinv = torch.empty(n, device=dev)
        prp, pci, pnnz = snaps[-1]
        dg.delta_rebuild(prp, pci, pnnz, ar, ac, int(ar.numel()), dr, dc, int(dr.numel()), rp, ci, dinv, ws_r)
        snaps.append((rp, ci, blk.nnz[t - 1]))
    cap = int(max(blk.nnz) * 1.6)
    bufs = [(torch.empty(n + 1, dtype=torch.int32, device=dev), torch.empty(cap, dtype=torch.int32, device=dev),
             torch.empty(cap, device=dev)) for _ in range(2)]
    ws = torch.empty(dg.csr_combine_workspace(cap), dtype=torch.uint8, device=dev)
    rows = []

    status = torch.zeros(1, dtype=torch.int32, device=dev)

    def series(record):
        s = (snaps[0][0], snaps[0][1], None, snaps[0][2])
        nnz_s = snaps[0][2]
        for t in range(2, blk.T + 1):
            out = bufs[t % 2]
            a_out = snaps[t - 1 - life] if t - life >= 1 else None
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            dg.csr_combine(s, snaps[t - 1], 1.0, a_out, -1.0, out, ws, diag_value=1.0, status=status)
            e1.record()
            torch.cuda.synchronize()
            nnz = int(out[0][n])                  # read back for the report only: the call itself never waits for it
            assert int(status) == 0
            if record:
                byts = 8 * nnz_s + 4 * snaps[t - 1][2] + (4 * a_out[2] if a_out else 0) + 8 * nnz + 4 * (n + 1) * (4 if a_out else 3)
                rows.append({"t": t, "nnz_s": nnz_s, "nnz_c": nnz, "ms": round(e0.elapsed_time(e1), 3),
                             "algorithmic_GBps": round(byts / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)})
            s, nnz_s = (out[0], out[1], out[2], cap), nnz    # downstream calls get the capacity as the upper bound
        return s

    series(False)
    s = series(True)
    dinv = torch.empty(n, device=dev)
    ws_d = torch.empty(dg.csr_weighted_dinv_workspace(s[3]), dtype=torch.uint8, device=dev)
    dg.csr_weighted_dinv(s[0], s[2], s[3], dinv, ws_d)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    dg.csr_weighted_dinv(s[0], s[2], s[3], dinv, ws_d)
    e1.record()
    torch.cuda.synchronize()
    out = {"edge_life": life, "steps": rows, "csr_weighted_dinv_ms": round(e0.elapsed_time(e1), 3),
           "note": "each step: a count launch, two small scans and a write launch, enqueue-only; the size of the result stays on the device"}
    del snaps, bufs, ws, s
    torch.cuda.empty_cache()
    progress("sliding-window sums timed")
    if args.smoothing_sum_only:
        return out
    # the whole forward pass on smoothed snapshots: rebuild, sliding-window sum, normalisation, X W, aggregation
    from paper_2109_07893_amd.pipeline import SmoothedRunner, StageTimer
    runner = SmoothedRunner(blk, life)
    runner.run_resident()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        runner.run_resident()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    # the same pass with rebuild, sliding-window sum, normalisation and X W of the next snapshot on a second stream
    runner.run_resident(overlap=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        runner.run_resident(overlap=True)
    torch.cuda.synchronize()
    ms_two = (time.perf_counter() - t0) / args.steps * 1e3
    runner.timer = StageTimer(dev)
    runner.run_resident()
    torch.cuda.synchronize()
    stored = runner.stored_entries()
    out["forward_pass"] = {"ms_per_step": round(ms, 3), "two_streams_ms_per_step": round(ms_two, 3),
                           "snapshots_per_step": blk.T, "stored_entries_last": stored,
                           "stages": {k: {"calls_per_step": c, "avg_ms": round(t / c, 4)}
                                      for k, (c, t) in runner.timer.totals().items()},
                           "note": "every snapshot t = 1..T, including the copy of A_1 into the ring at the start of the pass"}
    del runner
    torch.cuda.empty_cache()
    progress("pass on smoothed snapshots timed")
    # training step on the smoothed snapshots: every S_t (and S_t^T) stays resident, the backward pass does no graph work
    from dtdg_synth import gradient
    from paper_2109_07893_amd.training import make_smoothed_trainer
    # as many timesteps as fit beside the inputs: activations, M-transformed output and two gradient tensors per frame,
    # index and value arrays per smoothed snapshot (twice for a directed workload)
    free, _ = torch.cuda.mem_get_info(dev)
    per_t = 4 * blk.n * blk.f * blk.x[0].element_size() * max(blk.layers, 1) + 2 * 8 * int(max(blk.nnz) * 1.3)
    t_fit = max(2, min(blk.T, int(0.6 * free / per_t)))
    if t_fit < blk.T:
        from paper_2109_07893_amd.pipeline import BlockInputs
        blk = BlockInputs(n=blk.n, T=t_fit, f=blk.f, layers=blk.layers, window=blk.window, rowptr1=blk.rowptr1,
                          colidx1=blk.colidx1, deltas=blk.deltas[:t_fit - 1], x=blk.x[:t_fit], w=blk.w, nnz=list(blk.nnz[:t_fit]))
    tr = make_smoothed_trainer(wl, blk, life)
    g_y = torch.stack([gradient(wl, t, dev) for t in range(1, blk.T + 1)])
    tr.forward(); tr.backward(g_y)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        tr.forward(); tr.backward(g_y)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    tr.timer = StageTimer(dev)
    tr.forward(); tr.backward(g_y)
    torch.cuda.synchronize()
    out["training_step"] = {"ms_per_step": round(ms, 3), "snapshots_per_step": blk.T,
                            "stages": {k: {"calls_per_step": c, "avg_ms": round(t / c, 4)} for k, (c, t) in tr.timer.totals().items()}}
    return out


def cdgcn_layer(args, wl, blk, dev):
    """Forward pass of one CD-GCN layer over the block (every snapshot t = 1..T): an extra figure."""
    import math
    import torch
    from paper_2109_07893_amd.cdgcn import CdgcnLayer
    from paper_2109_07893_amd.pipeline import StageTimer
    f, hidden = blk.f, 32
    if 2 * f > 128:
        return {"skipped": f"the layer's concatenated output is {2 * f} wide; the dense transform takes widths up to 128"}
    dt = blk.x[0].dtype
    gen = torch.Generator(device=dev).manual_seed(wl.seed)
    w_x = (torch.randn((2 * f, 4 * hidden), generator=gen, device=dev) / math.sqrt(2 * f)).to(dt)
    w_h = (torch.randn((hidden, 4 * hidden), generator=gen, device=dev) / math.sqrt(hidden)).to(dt)
    bias = torch.zeros(4 * hidden, device=dev)
    layer = CdgcnLayer(blk, blk.w[0], w_x, w_h, bias, hidden)
    layer.load_first()
    for _ in range(max(1, args.warmup - 1)):
        layer.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        layer.run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    layer.timer = StageTimer(dev)
    layer.run()
    torch.cuda.synchronize()
    stages = {k: {"calls_per_step": c, "avg_ms": round(t / c, 4)} for k, (c, t) in layer.timer.totals().items()}
    edges = sum(blk.nnz)
    out = {"ms_per_step": ms, "value": edges / (ms * 1e-3), "unit": "edges/s", "hidden": hidden, "stages": stages,
           "what": f"t=1..{blk.T}: rebuild (t>=2), row scale, Y0 = A~ X, Y1 = Y0 W, relu(Y0 o Y1), "
                   "two gate products, LSTM cell"}
    # training step of the same layer: forward keeping (h_t, c_t), backward recomputing each timestep
    from paper_2109_07893_amd.cdgcn import CdgcnTrainer
    del layer
    torch.cuda.empty_cache()
    g_h = torch.randn((blk.T, blk.n, hidden), generator=gen, device=dev).to(dt)
    for key, keep in (("training_step", False), ("training_step_activations_kept", True)):
        tr = CdgcnTrainer(blk, blk.w[0], w_x, w_h, bias, hidden, keep_activations=keep)
        tr.load_first()
        tr.forward(); tr.backward(g_h)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            tr.forward(); tr.backward(g_h)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.steps * 1e3
        tr.timer = StageTimer(dev)
        tr.forward(); tr.backward(g_h)
        torch.cuda.synchronize()
        out[key] = {"ms_per_step": ms, "value": edges / (ms * 1e-3), "unit": "edges/s",
                    "stages": {k: {"calls_per_step": c, "avg_ms": round(t / c, 4)} for k, (c, t) in tr.timer.totals().items()},
                    "what": "forward keeping the LSTM states" + (", Y0 and Y" if keep else "") + "; backward " +
                            ("from the kept activations" if keep else "recomputing the GCN operation per timestep, reverse rebuilds") +
                            ", gate pre-activations recomputed; parameter gradients"}
        del tr
        torch.cuda.empty_cache()
    return out


def lstm_step_shapes(args, wl, blk, dev):
    """The fused LSTM step (gate pre-activations kept on chip) on every storage type and width it is built for,
    beside the same step composed of two dense transforms and the cell kernel: an extra figure, n rows of the
    workload, random inputs."""
    import math
    import torch
    import paper_2109_07893_amd as dg
    n = blk.n
    gen = torch.Generator(device=dev).manual_seed(wl.seed)
    rows = []
    for dt, hidden, f_y in ((torch.float32, 32, 64), (torch.float32, 16, 32), (torch.bfloat16, 32, 64), (torch.bfloat16, 64, 64),
                            (torch.bfloat16, 64, 128)):
        y = torch.randn((n, f_y), generator=gen, device=dev).to(dt)
        h = torch.randn((n, hidden), generator=gen, device=dev).to(dt)
        c = torch.randn((n, hidden), generator=gen, device=dev).to(dt)
        hn = torch.empty_like(h)
        w_x = (torch.randn((f_y, 4 * hidden), generator=gen, device=dev) / math.sqrt(f_y)).to(dt)
        w_h = (torch.randn((hidden, 4 * hidden), generator=gen, device=dev) / math.sqrt(hidden)).to(dt)
        bias = torch.zeros(4 * hidden, device=dev)
        gx = torch.empty((n, 4 * hidden), dtype=dt, device=dev)
        gh = torch.empty_like(gx)

        def fused():
            dg.lstm_step(y, h, w_x, w_h, bias, c, hn)

        def composed():
            dg.feature_transform(y, w_x, gx)
            dg.feature_transform(h, w_h, gh)
            dg.lstm_cell(gx, gh, bias, c, c, hn)

        ms = {"composed": None}
        for name, fn in (("fused", fused), ("composed", composed)):
            if name == "composed" and 4 * hidden > 128:      # the dense transform's widths end at 128
                continue
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms[name] = e0.elapsed_time(e1) / args.steps
        s = y.element_size()
        byts = s * n * (f_y + 4 * hidden)                  # Y, h, c in; c, h out
        flops = 2 * n * (f_y + hidden) * 4 * hidden
        rows.append({"dtype": "bf16" if dt == torch.bfloat16 else "f32", "hidden": hidden, "f_y": f_y,
                     "fused_ms": round(ms["fused"], 3), "composed_ms": None if ms["composed"] is None else round(ms["composed"], 3),
                     "fused_algorithmic_GBps": round(byts / (ms["fused"] * 1e-3) / 1e9, 1),
                     "fused_TFLOPs": round(flops / (ms["fused"] * 1e-3) / 1e12, 1)})
        del y, h, c, hn, gx, gh
        torch.cuda.empty_cache()
    return {"n": n, "shapes": rows}


def training_step(args, wl, blk, dev):
    """Forward keeping activations plus backward over the same block (every snapshot t = 1..T); an extra
    figure next to the headline, which stays the forward pass."""
    import torch
    from dtdg_synth import gradient
    from paper_2109_07893_amd.pipeline import StageTimer
    from paper_2109_07893_amd.training import make_trainer
    # The whole series in one block if its activations and gradients fit next to the inputs (the upstream
    # gradient and three more tensors of T x N x F); otherwise the paper's gradient checkpointing: blocks of
    # timesteps, a forward pass that keeps only the hand-over, then per block a rerun and the backward pass.
    from paper_2109_07893_amd.training import CheckpointedTrainer
    frame = blk.n * blk.f * blk.x[0].element_size()
    free_bytes, _ = torch.cuda.mem_get_info(dev)
    fit = int((0.85 * free_bytes - blk.T * frame) // (3 * frame))
    n_blocks = 1 if fit >= blk.T else -(-blk.T // max(fit, 2))
    g_y = torch.empty((blk.T, blk.n, blk.f), dtype=blk.x[0].dtype, device=dev)
    for t in range(1, blk.T + 1):
        g_y[t - 1].copy_(gradient(wl, t, device=dev))
    if n_blocks == 1:
        tr = make_trainer(wl, blk, keep_snapshots=getattr(args, "_keep_snapshots", False))
        timed = tr

        def one_step():
            tr.forward()
            tr.backward(g_y)
    else:
        ck = CheckpointedTrainer(wl, blk, -(-blk.T // n_blocks))
        timed = ck.trainer

        def one_step():
            ck.forward()
            ck.backward(g_y)
    directed = timed.directed
    progress(f"trainer ready ({n_blocks} block(s) of timesteps)")
    torch.cuda.synchronize()

    for _ in range(max(1, args.warmup - 1)):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    progress(f"training step timed: {ms:.2f} ms per step")
    timed.timer = StageTimer(dev)
    one_step()
    torch.cuda.synchronize()
    stages = {}
    for name, (calls, total_ms) in timed.timer.totals().items():
        if name in ("mproduct", "mproduct_backward"):
            byts = algorithmic_bytes(blk, name) / n_blocks          # a call mixes one block of the series
        elif name == "delta_rebuild":
            byts = None
        elif name in ("spmm", "spmm_transposed"):
            byts = sum(algorithmic_bytes(blk, name, t) for t in range(1, blk.T + 1)) / blk.T
        else:
            byts = algorithmic_bytes(blk, name, 1)
        entry = {"calls_per_step": calls, "avg_ms": round(total_ms / calls, 4), "ms_per_step": round(total_ms, 4)}
        if byts:
            entry["algorithmic_bytes_per_call"] = int(byts)
            entry["algorithmic_GBps"] = round(byts / (total_ms / calls * 1e-3) / 1e9, 1)
        stages[name] = entry
    edges = sum(blk.nnz)
    return {"ms_per_step": ms, "value": edges / (ms * 1e-3), "unit": "edges/s",
            "what": f"forward keeping activations + backward over t=1..{blk.T} ({'directed: second chain of transposed snapshots' if directed else 'undirected: the snapshot is its own transpose'}); "
                    "weight gradients of every layer, reverse rebuilds with exchanged lists"
                    + (f"; gradient checkpointing over {n_blocks} blocks: every block's forward pass runs twice" if n_blocks > 1 else ""),
            "checkpoint_blocks": n_blocks,
            "edges_per_step": edges, "stages": stages}


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (one GPU's block of timesteps, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2109_07893_amd as dg
    from dtdg_synth import WORKLOADS
    from dtdg_synth.blocks import make_block
    from paper_2109_07893_amd.pipeline import BlockRunner, StageTimer

    dg.load_library()
    wl = WORKLOADS[args.workload]
    if args.n:
        wl = wl.scaled(args.n)
    if args.natural_labels:
        from dataclasses import replace
        wl = replace(wl, scramble=False, name=wl.name + "-natural")
    T = args.T or wl.T
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    # c5 is defined with its difference lists in pinned host memory: the copies (dgnn_delta_h2d on a second stream,
    # one step ahead) are then inside the timed region.  The other workloads keep their lists in HBM.
    pinned = (args.workload == "c5" or args.pinned) and not args.resident
    t_gen = time.perf_counter()
    blk = make_block(wl, dev, gen_device=dev if args.gen_device == "cuda" else "cpu", pinned=pinned, T=T,
                     repeat_features=args.repeat_features, progress=progress)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    progress(f"inputs of {wl.name} generated in {t_gen:.1f} s")

    runner = BlockRunner(blk)
    runner.load_first()
    # Workloads without a window count only the snapshots that were rebuilt from a difference (t >= 2, A_1 is
    # sent whole outside the timed region); workloads with a window need every frame for the M-transform.
    first = 1 if blk.window else 2
    edges_per_step = sum(blk.nnz[first - 1:])

    settled = [0, 0]      # passes of the settle phase so far (-1 once it is over), and their final number

    def timed(step_fn, before=None, after=None):
        """Seconds per step of step_fn over args.steps back-to-back steps after args.warmup untimed ones."""
        if before:
            before()
        if settled[0] >= 0 and args.settle_seconds > 0:
            # preparation, like generating the inputs: one pass to learn how long it takes, then as many as fill the
            # settle time, enqueued back to back (a wait after every pass lets the device fall idle in between)
            t_settle = time.perf_counter()
            step_fn()
            torch.cuda.synchronize()
            one = max(time.perf_counter() - t_settle, 1e-4)
            more = min(int(args.settle_seconds / one), 1000)
            for _ in range(more):
                step_fn()
            torch.cuda.synchronize()
            settled[1] = 1 + more
        settled[0] = -1                                               # once: the later figures find the device warm
        for _ in range(args.warmup):
            step_fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_fn()
        torch.cuda.synchronize()
        el = (time.perf_counter() - t0) / args.steps
        if after:
            after()
        return el

    def resident_step():
        runner.run_resident(first=first)

    def pinned_step():            # steps follow one another: the first lists of the next step travel while this one finishes
        runner.run_from_pinned(first=first, prefetch_next=True)

    def pinned_single_block():    # a step on its own: its first copy has nothing to hide behind
        runner.run_from_pinned(first=first)

    if pinned:
        one_step = pinned_step
        per_step = timed(pinned_step)
        runner.run_from_pinned(first=first)          # consumes the outstanding request
        torch.cuda.synchronize()
    else:
        one_step = resident_step
        per_step = timed(resident_step)
    ms_per_step = per_step * 1e3
    value = edges_per_step / per_step
    progress(f"forward timed: {ms_per_step:.2f} ms per step ({'pinned host lists' if pinned else 'lists resident'})")

    # per-stage durations: the same steps again with an event pair around every library call, on the stream it is
    # enqueued on (the list copies on the copy stream)
    runner.timer = StageTimer(dev)
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    totals = runner.timer.totals()
    runner.timer = None
    if pinned:
        runner.run_from_pinned(first=first)
        torch.cuda.synchronize()
    stages = {}
    for name, (calls, ms) in totals.items():
        per_step_calls = calls // args.steps
        if name == "mproduct":
            byts = algorithmic_bytes(blk, name)
        elif name == "delta_h2d":
            byts = sum(8 * (d[0].numel() + d[2].numel()) for d in blk.deltas) / max(per_step_calls, 1)
        else:
            ts = range(2, T + 1) if name == "delta_rebuild" else range(first, T + 1)
            reps = blk.layers if name in ("feature_transform", "spmm") else 1
            byts = sum(algorithmic_bytes(blk, name, t) for t in ts) * reps / max(per_step_calls, 1)
        avg_ms = ms / calls
        stages[name] = {"calls_per_step": per_step_calls, "avg_ms": round(avg_ms, 4),
                        "ms_per_step": round(ms / args.steps, 4), "algorithmic_bytes_per_call": int(byts),
                        "algorithmic_GBps": round(byts / (avg_ms * 1e-3) / 1e9, 1)}
        if name == "delta_h2d":
            stages[name]["note"] = "host link (PCIe), on the copy stream, overlapped with the other stages; not HBM traffic"
    on_gpu = {k: v for k, v in stages.items() if k != "delta_h2d"}
    dominant = max(on_gpu, key=lambda k: on_gpu[k]["ms_per_step"])
    achieved = stages[dominant]["algorithmic_GBps"]
    kernels = {"spmm": "dgnn_spmm (spmm_stream_kernel + spmm_carry_kernel)",
               "delta_rebuild": "dgnn_delta_rebuild (rowptr_kernel + merge_kernel)",
               "feature_transform": "dgnn_feature_transform (xw kernel)", "mproduct": "dgnn_mproduct (mproduct_kernel)"}
    traffic, traffic_note = committed_traffic(args.workload, dominant)
    roofline = {"bound": "hbm", "kernel": kernels[dominant], "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_note,
                "avg_ms": stages[dominant]["avg_ms"],
                "algorithmic_bytes_per_call": stages[dominant]["algorithmic_bytes_per_call"]}
    if traffic:   # counter bytes of the committed profile (taken on the same kernel source) over the duration measured now
        roofline["traffic_l2_miss_GBps"] = round(traffic / (stages[dominant]["avg_ms"] * 1e-3) / 1e9, 1)
        roofline["traffic_note"] = ("FETCH_SIZE / WRITE_SIZE count what leaves the L2s: fetches served by the Infinity Cache are "
                                    "included, so the rate is L2-miss traffic, not an HBM fraction")
    all_bytes = sum(v["algorithmic_bytes_per_call"] * v["calls_per_step"] for v in on_gpu.values())

    lists_where = ("pinned host memory; dgnn_delta_h2d on a second stream inside the timed region, one step ahead; steps "
                   "follow one another, so the first lists of the next step are requested while this one finishes"
                   if pinned else "resident in HBM")
    out = {
        "metric": "snapshot-edges/sec (delta rebuild + SpMM)", "value": value, "unit": "edges/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "settle_steps_before_warmup": settled[1], "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if wl.dtype == "f32" else "bf16 storage, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: N={blk.n}, T={T}, {wl.graph}, F={blk.f}, {wl.dtype}, layers={blk.layers}, "
                               f"window={blk.window}, churn del {wl.del_frac:g} + add {wl.add_frac:g} per step",
                   "snapshots_per_step": T - first + 1, "edges_per_step": edges_per_step,
                   "nnz_first": blk.nnz[0], "nnz_last": blk.nnz[-1], "difference_lists": lists_where,
                   "timed": f"t={first}..{T}: " + ("list copy host -> device + " if pinned else "")
                            + ("delta rebuild (t>=2) + " if first == 1 else "delta rebuild + ")
                            + f"{blk.layers}x(X W + SpMM)" + (" + M-transform" if blk.window else "")},
        "roofline": roofline,
        "stages": stages,
        "hbm_frac_algorithmic_whole_step": round(all_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "north_star_target": {"hbm_frac": 0.60, "met": bool(all_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS >= 0.60),
                              "note": "target: delta rebuild + SpMM at 60 % of the HBM peak; the fractions above count "
                                      "algorithmic bytes (every row of H fetched once), the gather of a scrambled power-law "
                                      "graph moves several times that"},
        "generate_s": round(t_gen, 2),
    }

    if pinned:
        el_single = timed(pinned_single_block)
        el_res = timed(resident_step)
        h2d = sum(8 * (d[0].numel() + d[2].numel()) for d in blk.deltas)
        # the copies alone, nothing computing: what the host link delivers for these list sizes
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for lists in blk.pinned:
            dg.delta_h2d(*lists, *runner.stage[0])
        torch.cuda.synchronize()
        link_s = time.perf_counter() - t0
        out["pinned_host_lists"] = {"h2d_bytes_per_step": h2d, "h2d_alone_ms": link_s * 1e3, "h2d_alone_GBps": h2d / link_s / 1e9,
                                    "single_block": {"value": edges_per_step / el_single, "unit": "edges/s", "ms_per_step": el_single * 1e3,
                                                     "note": "one step on its own: the first copy of the step is not hidden"},
                                    "whole_snapshot_bytes_per_step": sum(4 * (z + blk.n + 1) for z in blk.nnz[1:])}
        out["lists_resident_in_hbm"] = {"value": edges_per_step / el_res, "unit": "edges/s", "ms_per_step": el_res * 1e3,
                                        "note": "the same step without the host-to-device copies (not the headline)"}

    progress("per-stage pass done")
    if args.graph:
        graph = runner.capture(first=first)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        el = (time.perf_counter() - t0) / args.steps
        out["hip_graph_replay"] = {"value": edges_per_step / el, "unit": "edges/s", "ms_per_step": el * 1e3}
        del graph
        progress("graph replay timed")
        if not args.no_train:
            # the training step (forward + backward over every snapshot) as one graph, if it fits in one block
            try:
                from dtdg_synth import gradient
                from paper_2109_07893_amd.training import capture_training_step, make_trainer
                g_y = torch.stack([gradient(wl, t, dev) for t in range(1, blk.T + 1)])
                tr = make_trainer(wl, blk)
                tgraph = capture_training_step(tr, g_y)
                tgraph.replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    tgraph.replay()
                torch.cuda.synchronize()
                el = (time.perf_counter() - t0) / args.steps
                out["hip_graph_replay"]["training_step"] = {"value": sum(blk.nnz) / el, "unit": "edges/s", "ms_per_step": el * 1e3}
                del tgraph, tr, g_y
            except Exception as exc:                  # noqa: BLE001 -- an extra figure (a large workload may not fit twice)
                out["hip_graph_replay"]["training_step"] = {"error": f"{type(exc).__name__}: {exc}"[:300]}
            torch.cuda.empty_cache()
    # figures of the rows built after the hot path: on request, or all of them unless --no-extras; a failure there is
    # reported in its own object and never costs the headline line
    def extra(key, flag, fn):
        if not (flag or not args.no_extras):
            return
        try:
            out[key] = fn(args, wl, blk, dev)
        except Exception as exc:                      # noqa: BLE001 -- reported, the headline still goes out
            out[key] = {"error": f"{type(exc).__name__}: {exc}"[:300]}
        torch.cuda.empty_cache()
        progress(f"{key} timed")

    extra("two_streams", args.two_streams, two_stream_steps)
    extra("gather_working_sets", args.working_sets, gather_working_sets)
    extra("mproduct_explicit_band", args.mproduct_band, mproduct_band)
    extra("cdgcn_layer", args.cdgcn, cdgcn_layer)
    extra("lstm_step_shapes", args.cdgcn, lstm_step_shapes)
    extra("weighted_step", args.weighted, weighted_step)
    extra("smoothing", args.smoothing, smoothing_steps)
    if not args.no_train:
        del runner
        torch.cuda.empty_cache()
        out["training_step"] = training_step(args, wl, blk, dev)
        if out["training_step"].get("checkpoint_blocks", 1) == 1:
            # the same step with every snapshot of the block resident (no reverse rebuilds on the way back)
            torch.cuda.empty_cache()
            args._keep_snapshots = True
            try:
                kept = training_step(args, wl, blk, dev)
                out["training_step_snapshots_kept"] = {k: kept[k] for k in ("ms_per_step", "value", "unit") if k in kept}
            except Exception as exc:                  # noqa: BLE001 -- an extra figure
                out["training_step_snapshots_kept"] = {"error": f"{type(exc).__name__}: {exc}"[:300]}
            args._keep_snapshots = False

    if not args.no_cpu_baseline:
        progress("timing the CPU oracle")
        out["cpu_baseline"] = cpu_baseline(wl, blk, first, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
