#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--no-cpu] [--no-all]

One step = encode the database rows (bundle layout) + encode the queries + exhaustive
top-K search, all through the C-ABI library, with the fp32 inputs already resident in
HBM.  Prints ONE JSON line: queries/s of the whole step on the headline workload, the
roofline position of the dominant kernel (the XOR + population-count scan, timed with HIP
events inside the library on the stream it runs on), the few-query regime the paper
measures, the same step on the other workloads (``all_workloads``), and the CPU oracle
timed on the host cores.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def source_sha16() -> str:
    """Fingerprint of the kernel and host sources of the library (csrc/): the profile summaries
    under profiles/ carry the fingerprint of the sources they were taken from, so a figure that
    comes from a stale profile shows."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2008_02002_amd", "csrc")
    for name in sorted(f for f in os.listdir(csrc) if f.endswith((".hip", ".h"))):
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def cpu_baseline(w, bits, db_bits, k, scale, budget_s=15.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the same
    workload: the whole database is encoded and the first q queries are searched, q
    sized from a short probe so the search takes about budget_s seconds."""
    from oracle import scale as oc
    from paper_2008_02002_amd import workloads as wl

    X = wl.database(w)
    t0 = time.perf_counter()
    planes = oc.encode(X, db_bits, scale)
    t_enc = time.perf_counter() - t0
    del X
    Q = wl.queries(w)
    qplanes = oc.encode(Q, bits, scale)
    probe = min(w.m, 4 * oc.threads())
    t0 = time.perf_counter()
    oc.search(planes, qplanes[:probe], w.d, k)
    t_probe = time.perf_counter() - t0
    q = int(min(w.m, max(probe, budget_s / max(t_probe, 1e-6) * probe)))
    t0 = time.perf_counter()
    oc.search(planes, qplanes[:q], w.d, k)
    t_search = time.perf_counter() - t0
    whole_job = t_enc + t_search * (w.m / q)
    return {
        "value": w.m / whole_job,
        "unit": "queries/s",
        "cores": oc.threads(),
        "kind": "oracle",
        "sample": (f"database of {w.n} rows encoded in {t_enc:.2f}s; first {q} of {w.m} queries searched "
                   f"over all rows in {t_search:.2f}s; whole job extrapolated linearly in the query count"),
    }


def exact_topk(Xdb_dev, Xq_dev, k, slab_bytes=1 << 28):
    """Exact fp32 cosine top-K rows per query.  The similarity matrix is produced in row slabs
    whose outputs stay far below 2 GiB (one matmul with a larger output returned wrong values on
    this software stack), each slab's top-K is kept, and the slab winners are merged."""
    import torch
    nq, n = Xq_dev.shape[0], Xdb_dev.shape[0]
    slab = max(k, slab_bytes // (4 * nq))
    vals, rows = [], []
    for lo in range(0, n, slab):
        hi = min(n, lo + slab)
        v, i = torch.topk(Xq_dev @ Xdb_dev[lo:hi].T, min(k, hi - lo), dim=1)
        vals.append(v)
        rows.append(i + lo)
    vals, rows = torch.cat(vals, dim=1), torch.cat(rows, dim=1)
    best = torch.topk(vals, k, dim=1).indices
    return torch.gather(rows, 1, best)


def recall_at_k(Xdb_dev, Xq_dev, idx_dev, k, nq=256):
    """Precision@K (Section 5) of the returned rows against exact fp32 cosine, first nq queries."""
    nq = min(nq, Xq_dev.shape[0], idx_dev.shape[0])
    real = exact_topk(Xdb_dev, Xq_dev[:nq], k)
    hits = 0
    for i in range(nq):
        hits += len(set(real[i].tolist()) & set(idx_dev[i].tolist()))
    return hits / float(nq * k), nq


def fp32_reference_error(Xdb_dev, Xq_dev, nq=16, rows=100_000):
    """Largest absolute difference between the fp32 cosine matrix the recall figure is taken
    against and the same products in float64, on the first nq queries x first `rows` rows."""
    nq = min(nq, Xq_dev.shape[0])
    rows = min(rows, Xdb_dev.shape[0])
    s32 = Xq_dev[:nq] @ Xdb_dev[:rows].T
    s64 = Xq_dev[:nq].double() @ Xdb_dev[:rows].double().T
    return float((s32.double() - s64).abs().max())


def recall_by_scale(xbq, wl, w, Xdb, Xq, bits, db_bits, k, nq=256):
    """Recall of the plain search at the three scale choices of Section 3.6: none (1), the
    conservative 1 / max|x| and the relaxed 1 / (98th percentile of |x|)."""
    import torch
    nq = min(nq, w.m)
    head = wl.database(w, 0, min(w.n, 100_000))
    scales = {"1": 1.0, "1/max": wl.choose_scale(head, 1.0), "1/q98": wl.choose_scale(head, 0.98)}
    db = torch.empty(xbq.xbq_code_bytes(w.n, w.d, db_bits, xbq.BUNDLE64) // 4, dtype=torch.int32, device="cuda")
    q = torch.empty(xbq.xbq_code_bytes(nq, w.d, bits, xbq.ROWS) // 4, dtype=torch.int32, device="cuda")
    ws = torch.empty(xbq.xbq_search_workspace_bytes(w.n, nq, w.d, bits, k), dtype=torch.uint8, device="cuda")
    idx = torch.empty((nq, k), dtype=torch.int32, device="cuda")
    score = torch.empty((nq, k), dtype=torch.int32, device="cuda")
    out = {}
    for name, s in scales.items():
        xbq.xbq_encode(Xdb, db_bits, s, xbq.BUNDLE64, out=db)
        xbq.xbq_encode(Xq[:nq], bits, s, xbq.ROWS, out=q)
        xbq.xbq_search_asym(db, w.n, db_bits, q, nq, bits, w.d, k, workspace=ws, idx=idx, score=score)
        torch.cuda.synchronize()
        out[name] = {"scale": s, "recall": recall_at_k(Xdb, Xq, idx, k, nq)[0]}
    return out


def resident_inputs(wl, w):
    """fp32 database and queries of a workload in HBM (generated in slabs of 2^20 rows)."""
    import torch
    Xq = torch.from_numpy(wl.queries(w)).cuda()
    Xdb = torch.empty((w.n, w.d), dtype=torch.float32, device="cuda")
    slab = 1 << 20
    for lo in range(0, w.n, slab):
        hi = min(w.n, lo + slab)
        Xdb[lo:hi] = torch.from_numpy(wl.database(w, lo, hi)).cuda()
    return Xdb, Xq


def timed_steps(xbq, Xdb, Xq, db, q, w, bits, db_bits, scale, search, steps, warmup):
    """W untimed and K timed steps (encode database, encode queries, search); returns the
    step time, the summed scan-kernel time of the timed steps (HIP events inside the library,
    on the stream the kernels run on) and the database-encode time."""
    import torch

    def step():
        xbq.xbq_encode(Xdb, db_bits, scale, xbq.BUNDLE64, out=db)
        xbq.xbq_encode(Xq, bits, scale, xbq.ROWS, out=q)
        search()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    xbq.xbq_trace_enable(True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    enc_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        enc_ev[i][0].record()
        xbq.xbq_encode(Xdb, db_bits, scale, xbq.BUNDLE64, out=db)
        enc_ev[i][1].record()
        xbq.xbq_encode(Xq, bits, scale, xbq.ROWS, out=q)
        search()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = e0.elapsed_time(e1)
    scan_ms, launches, pairs = xbq.xbq_trace_read()
    xbq.xbq_trace_enable(False)
    enc_ms = sum(a.elapsed_time(b) for a, b in enc_ev) / steps
    return {"ms_per_step": max(wall_ms, gpu_ms) / steps, "scan_ms": scan_ms, "launches": launches, "pairs": pairs,
            "enc_ms": enc_ms}


def few_queries_leg(xbq, cm, w, Xdb, Xq, db, q, bits, db_bits, k, mq, reps=30):
    """The regime the paper measured (Section 5: single-query requests): mq queries against the
    resident codes.  One query is bound by the HBM stream of the database codes; from about three
    queries on the vector ALUs bind (both fractions are reported)."""
    import torch
    idx1 = torch.empty((mq, k), dtype=torch.int32, device="cuda")
    sc1 = torch.empty((mq, k), dtype=torch.int32, device="cuda")
    wsb = xbq.xbq_search_workspace_bytes(w.n, mq, w.d, bits, k)
    ws1 = torch.empty(wsb, dtype=torch.uint8, device="cuda")

    def one():
        xbq.xbq_search_asym(db, w.n, db_bits, q, mq, bits, w.d, k, workspace=ws1, idx=idx1, score=sc1)

    for _ in range(3):
        one()
    torch.cuda.synchronize()
    # request latency, calls back to back; timed without the library's scan trace, whose event
    # records between the launches of a request add several microseconds to it
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a0.record()
    for _ in range(reps):
        one()
    a1.record()
    torch.cuda.synchronize()
    lat_ms = a0.elapsed_time(a1) / reps
    # the scan launches alone, from HIP events around them inside the library
    xbq.xbq_trace_enable(True)
    for _ in range(3):
        one()
    torch.cuda.synchronize()
    xbq.xbq_trace_read()                                # warm-up of the traced form, discarded
    for _ in range(reps):
        one()
    torch.cuda.synchronize()
    sms, sl, _ = xbq.xbq_trace_read()
    xbq.xbq_trace_enable(False)
    # the same search captured once in a HIP graph and replayed (no launch gaps from the host)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one()
    graph.replay()
    torch.cuda.synchronize()
    g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    g0.record()
    for _ in range(reps):
        graph.replay()
    g1.record()
    torch.cuda.synchronize()
    graph_ms = g0.elapsed_time(g1) / reps
    del graph
    # Algorithm 1 in full for the same queries (extra distance 100, fp32 refine), the request
    # the paper times: xbq_k_select on resident codes and resident fp32 rows
    ks_cap = min(w.n, 8192)
    ks_ws = torch.empty(xbq.lib().xbq_k_select_workspace_bytes(w.n, mq, w.d, bits, k, 100, ks_cap),
                        dtype=torch.uint8, device="cuda")
    ks_sim = torch.empty((mq, k), dtype=torch.float32, device="cuda")
    ks_cnt = torch.empty((mq,), dtype=torch.int32, device="cuda")

    def ksel():
        xbq.xbq_k_select(Xdb, db, db_bits, Xq[:mq], q, bits, k, 100, ks_cap, workspace=ks_ws, idx=idx1, sim=ks_sim,
                         cand=ks_cnt)

    for _ in range(3):
        ksel()
    torch.cuda.synchronize()
    k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    k0.record()
    for _ in range(reps):
        ksel()
    k1.record()
    torch.cuda.synchronize()
    ks_ms = k0.elapsed_time(k1) / reps
    scan_s = sms / reps * 1e-3
    code_bytes = w.n * cm.code_bytes_per_row(w.d, db_bits) * (sl / reps)          # one pass over the codes per scan launch
    stored = wsb >= 4 * w.n * mq                       # the selection over stored distances also writes 4 bytes per pair
    stream_bytes = code_bytes + (4 * w.n * mq if stored else 0)
    lane_ops = cm.credited_lane_ops_per_pair(w.d, bits, db_bits) * w.n * mq
    return {
        "queries": mq, "search_ms": lat_ms, "queries_per_s": mq / (lat_ms * 1e-3),
        "graph_replay_ms": graph_ms, "graph_queries_per_s": mq / (graph_ms * 1e-3),
        "k_select_extra100_ms": ks_ms, "k_select_mean_candidates": float(ks_cnt.float().mean()),
        "request_GBps": code_bytes / 1e9 / (lat_ms * 1e-3),
        "request_hbm_frac": code_bytes / (lat_ms * 1e-3) / cm.HBM_BYTES_PER_S,
        "scan_kernel_ms": sms / reps, "scan_launches": sl / reps,
        "scan_GBps": stream_bytes / 1e9 / scan_s,
        "scan_hbm_frac": stream_bytes / scan_s / cm.HBM_BYTES_PER_S,
        "scan_alu_frac": lane_ops / scan_s / cm.VALU_INT_LANE_OPS_PER_S,
        "hbm_floor_ms": code_bytes / cm.HBM_BYTES_PER_S * 1e3,
        "alu_floor_ms": lane_ops / cm.VALU_INT_LANE_OPS_PER_S * 1e3,
        "path": "selection over stored distances" if stored else "selection while the rows stream (nothing stored)",
        "note": "codes resident, encode not included; search_ms is the request (all its launches) back to back; "
                "scan time from HIP events around the scan launch in a second, traced loop (the event records add "
                "a few microseconds to a launch this short)"}


def ordered_rows_leg(xbq, wl, bits=4, k=100):
    """What the order of the rows costs: the same mixture (1 M x 128, 1000 clusters) with its rows
    shuffled and lying cluster by cluster; 10 000 queries in one call, and single-query requests."""
    import torch
    n, d, m = 1_000_000, 128, 10_000
    out = {"rows": f"{n} x {d}, Gaussian mixture of 1000 clusters (spread 0.25), {bits}-bit, K={k}"}
    for name, ordered in (("shuffled", False), ("by_cluster", True)):
        X, Q = wl.clustered_rows(n, d, m, 1000, 0.25, 11, ordered)
        db = xbq.xbq_encode(torch.from_numpy(X).cuda(), bits, 2.0, xbq.BUNDLE64)
        q = xbq.xbq_encode(torch.from_numpy(Q).cuda(), bits, 2.0, xbq.ROWS)
        del X, Q
        ws = torch.empty(xbq.xbq_search_workspace_bytes(n, m, d, bits, k), dtype=torch.uint8, device="cuda")
        idx = torch.empty((m, k), dtype=torch.int32, device="cuda")
        sc = torch.empty_like(idx)
        xbq.xbq_search(db, n, q, m, d, bits, k, workspace=ws, idx=idx, score=sc)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            xbq.xbq_search(db, n, q, m, d, bits, k, workspace=ws, idx=idx, score=sc)
        e1.record()
        torch.cuda.synchronize()
        batched_ms = e0.elapsed_time(e1) / 3
        W = (d + 31) // 32
        lat = []
        for i in range(16):                              # sixteen different single-query requests
            qi = q[i * bits * W:(i + 1) * bits * W]
            for _ in range(2):
                xbq.xbq_search(db, n, qi, 1, d, bits, k, workspace=ws, idx=idx[:1], score=sc[:1])
            torch.cuda.synchronize()
            e0.record()
            for _ in range(10):
                xbq.xbq_search(db, n, qi, 1, d, bits, k, workspace=ws, idx=idx[:1], score=sc[:1])
            e1.record()
            torch.cuda.synchronize()
            lat.append(e0.elapsed_time(e1) / 10)
        lat.sort()
        out[name] = {"search_10000_queries_ms": batched_ms, "one_query_median_ms": lat[len(lat) // 2],
                     "one_query_max_ms": lat[-1]}
        del db, q, ws, idx, sc
        torch.cuda.empty_cache()
    return out


def workload_summary(xbq, cm, wl, name, bits, k, steps, warmup):
    """One line of all_workloads: the same step as the headline on another workload."""
    import torch
    w = wl.WORKLOADS[name]
    scale = wl.workload_scale(w)
    Xdb, Xq = resident_inputs(wl, w)
    db = torch.empty(xbq.xbq_code_bytes(w.n, w.d, bits, xbq.BUNDLE64) // 4, dtype=torch.int32, device="cuda")
    q = torch.empty(xbq.xbq_code_bytes(w.m, w.d, bits, xbq.ROWS) // 4, dtype=torch.int32, device="cuda")
    ws = torch.empty(xbq.xbq_search_workspace_bytes(w.n, w.m, w.d, bits, k), dtype=torch.uint8, device="cuda")
    idx = torch.empty((w.m, k), dtype=torch.int32, device="cuda")
    score = torch.empty((w.m, k), dtype=torch.int32, device="cuda")

    def search():
        xbq.xbq_search_asym(db, w.n, bits, q, w.m, bits, w.d, k, workspace=ws, idx=idx, score=score)

    t = timed_steps(xbq, Xdb, Xq, db, q, w, bits, bits, scale, search, steps, warmup)
    ops = cm.credited_lane_ops_per_pair(w.d, bits, bits) * t["pairs"]
    enc_bytes = w.n * cm.encode_bytes_per_row(w.d, bits)
    out = {"workload": f"{w.name}: n={w.n} d={w.d} m={w.m} bits={bits} K={k}", "steps": steps, "warmup": warmup,
           "queries_per_s": w.m / (t["ms_per_step"] * 1e-3), "ms_per_step": t["ms_per_step"],
           "scan_ms_per_step": t["scan_ms"] / steps, "scan_launches_per_step": t["launches"] / steps,
           "scan_alu_frac": ops / (t["scan_ms"] * 1e-3) / cm.VALU_INT_LANE_OPS_PER_S,
           "encode_db_ms": t["enc_ms"], "encode_hbm_frac": enc_bytes / (t["enc_ms"] * 1e-3) / cm.HBM_BYTES_PER_S}
    if w.n * w.d <= 1 << 31:                             # the large ones would double the run for one more figure
        out["recall_at_k"] = recall_at_k(Xdb, Xq, idx, k)[0]
    one = few_queries_leg(xbq, cm, w, Xdb, Xq, db, q, bits, bits, k, 1, reps=10)
    out["one_query"] = {key: one[key] for key in ("search_ms", "request_hbm_frac", "graph_replay_ms", "scan_kernel_ms",
                                                   "scan_hbm_frac", "k_select_extra100_ms")}
    del Xdb, Xq, db, q, ws, idx, score
    torch.cuda.empty_cache()
    return out


ALL_WORKLOADS = (("C1", 4, 10, 20), ("C3", 3, 10, 3), ("C3", 4, 10, 3), ("C4", 3, 10, 3), ("C4", 3, 100, 3),
                 ("C5", 4, 100, 3))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--bits", type=int, default=0)
    ap.add_argument("--k", type=int, default=0)
    ap.add_argument("--db-bits", type=int, default=0, help="narrower database codes (xbq_search_asym)")
    ap.add_argument("--queries", type=int, default=0, help="use only the first N queries")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-recall", action="store_true")
    ap.add_argument("--no-all", action="store_true", help="skip the all_workloads leg (the other workloads)")
    ap.add_argument("--no-few", action="store_true", help="skip the few-query and cross-check legs")
    ap.add_argument("--no-ordered", action="store_true", help="skip the leg that compares shuffled rows with rows ordered by cluster")
    ap.add_argument("--refine", type=int, default=-1, metavar="EXTRA",
                    help="time the candidate search + fp32 refine (xbq_search_refine) with this extra distance")
    ap.add_argument("--k-select", type=int, default=-1, metavar="EXTRA",
                    help="time Algorithm 1 with the whole candidate list (xbq_k_select) with this extra distance")
    ap.add_argument("--max-candidates", type=int, default=1 << 17, help="candidate bound of --k-select")
    ap.add_argument("--calib-copy", action="store_true",
                    help="run one 256 MiB device-to-device copy first (reference for HBM byte counters)")
    ap.add_argument("--set", action="append", default=[], metavar="NAME=VALUE",
                    help="library tuning option (xbq_set_option), e.g. --set growth=4")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one process, one device, no collectives); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2008_02002_amd import costmodel as cm
    from paper_2008_02002_amd import workloads as wl
    from paper_2008_02002_amd import xbq

    w = wl.WORKLOADS[args.workload]
    if args.queries:
        w = wl.scaled_down(w, m=args.queries)
    bits = args.bits or w.bits[-1]
    db_bits = args.db_bits or bits
    k = args.k or w.ks[-1]
    torch.cuda.set_device(0)
    xbq.lib()
    for kv in args.set:
        name, value = kv.split("=")
        xbq.xbq_set_option(name, float(value))

    scale = wl.workload_scale(w)
    Xdb, Xq = resident_inputs(wl, w)
    db = torch.empty(xbq.xbq_code_bytes(w.n, w.d, db_bits, xbq.BUNDLE64) // 4, dtype=torch.int32, device="cuda")
    q = torch.empty(xbq.xbq_code_bytes(w.m, w.d, bits, xbq.ROWS) // 4, dtype=torch.int32, device="cuda")
    if args.k_select >= 0 and args.refine >= 0:
        sys.exit("bench.py: --refine and --k-select exclude each other")
    if args.k_select >= 0:
        wsb = xbq.lib().xbq_k_select_workspace_bytes(w.n, w.m, w.d, bits, k, args.k_select, args.max_candidates)
        sim = torch.empty((w.m, k), dtype=torch.float32, device="cuda")
        ncand = torch.empty((w.m,), dtype=torch.int32, device="cuda")
    elif args.refine >= 0:
        wsb = xbq.lib().xbq_search_refine_workspace_bytes(w.n, w.m, w.d, bits, k)
        sim = torch.empty((w.m, k), dtype=torch.float32, device="cuda")
        ncand = torch.empty((w.m,), dtype=torch.int32, device="cuda")
    else:
        wsb = xbq.xbq_search_workspace_bytes(w.n, w.m, w.d, bits, k)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    idx = torch.empty((w.m, k), dtype=torch.int32, device="cuda")
    score = torch.empty((w.m, k), dtype=torch.int32, device="cuda")

    def search():
        if args.k_select >= 0:
            xbq.xbq_k_select(Xdb, db, db_bits, Xq, q, bits, k, args.k_select, args.max_candidates, workspace=ws,
                             idx=idx, sim=sim, cand=ncand)
        elif args.refine >= 0:
            xbq.xbq_search_refine(Xdb, db, db_bits, Xq, q, bits, k, args.refine, workspace=ws, idx=idx, sim=sim,
                                  cand=ncand)
        else:
            xbq.xbq_search_asym(db, w.n, db_bits, q, w.m, bits, w.d, k, workspace=ws, idx=idx, score=score)

    if args.calib_copy:
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.int32, device="cuda")      # 256 MiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    t = timed_steps(xbq, Xdb, Xq, db, q, w, bits, db_bits, scale, search, args.steps, args.warmup)
    ms_per_step, scan_ms, launches, pairs, enc_ms = t["ms_per_step"], t["scan_ms"], t["launches"], t["pairs"], t["enc_ms"]

    ops = cm.credited_lane_ops_per_pair(w.d, bits, db_bits) * pairs          # credited XOR + popcount lane-ops
    achieved = ops / (scan_ms * 1e-3) / 1e12
    peak = cm.VALU_INT_LANE_OPS_PER_S / 1e12
    # HBM-side bytes per scan launch come from the committed rocprofv3 --pmc summary of this
    # same command (they cannot be read from inside the process); the summary carries the
    # fingerprint of the sources it was taken from, reported beside the figure
    here = source_sha16()
    traffic, traffic_sha = None, None
    tpath = os.path.join(ROOT, "profiles", f"bench_{w.name}.md")
    if os.path.exists(tpath) and not args.queries:
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_scan_launch:"):
                traffic = float(line.split(":")[1])
            if line.startswith("source_sha16:"):
                traffic_sha = line.split(":")[1].strip()
    # what the chip sustains on the streams the rooflines are about (register-only XOR +
    # population count; a streaming read of the fp32 database; a bare kernel with the encoder's
    # traffic mix), beside the published peaks
    pe0, pe1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    pout, pops = xbq.xbq_probe_valu(20000)
    torch.cuda.synchronize()
    pe0.record()
    xbq.xbq_probe_valu(20000, out=pout)
    pe1.record()
    torch.cuda.synchronize()
    valu_measured = pops / (pe0.elapsed_time(pe1) * 1e-3) / 1e12
    xbq.xbq_probe_read(Xdb, out=pout)
    torch.cuda.synchronize()
    pe0.record()
    for _ in range(5):
        xbq.xbq_probe_read(Xdb, out=pout)
    pe1.record()
    torch.cuda.synchronize()
    read_measured = 5 * Xdb.numel() * 4 / (pe0.elapsed_time(pe1) * 1e-3)
    enc_bytes = w.n * cm.encode_bytes_per_row(w.d, db_bits)
    mix_measured = None
    if w.d % 4 == 0:
        xbq.xbq_probe_encode_traffic(Xdb, db_bits, db)
        torch.cuda.synchronize()
        pe0.record()
        for _ in range(5):
            xbq.xbq_probe_encode_traffic(Xdb, db_bits, db)
        pe1.record()
        torch.cuda.synchronize()
        mix_measured = 5 * enc_bytes / (pe0.elapsed_time(pe1) * 1e-3)
        xbq.xbq_encode(Xdb, db_bits, scale, xbq.BUNDLE64, out=db)          # the probe overwrote the codes
        torch.cuda.synchronize()
    del pout

    out = {
        "metric": "queries/s, 1M x d128 4-bit K=100 (encode + XOR/popcount scan + top-K)"
                  if w.name == "C2" else f"queries/s, {w.name}",
        "value": w.m / (ms_per_step * 1e-3),
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "source_sha16": here,
        "config": {"workload": f"{w.name}: n={w.n} d={w.d} m={w.m} bits={bits}" +
                               (f"x{db_bits}" if db_bits != bits else "") + f" K={k} ({w.kind}, seed {w.seed})",
                   "scale": scale, "options": args.set,
                   "path": ("xbq_k_select extra=%d max_candidates=%d" % (args.k_select, args.max_candidates)
                            if args.k_select >= 0 else
                            "xbq_search_refine extra=%d" % args.refine if args.refine >= 0 else "xbq_search")},
        "roofline": {
            "bound": "alu",
            "kernel": "scan (XOR + population count), all launches of one step",
            "achieved": achieved,
            "peak": peak,
            "unit": "T lane-op/s (32-bit integer)",
            "frac": achieved / peak,
            "traffic": traffic,
            "traffic_from": None if traffic is None else {
                "file": f"profiles/bench_{w.name}.md", "source_sha16": traffic_sha,
                "sources_unchanged_since": traffic_sha == here},
            "measured_peak": valu_measured,
            "frac_of_measured_peak": achieved / valu_measured,
            "scan_ms_per_step": scan_ms / args.steps,
            "launches_per_step": launches / args.steps,
            "avg_launch_ms": scan_ms / max(launches, 1),
            # the batched scan is not an HBM stream: the codes are read about once per step
            "scan_code_GBps": w.n * cm.code_bytes_per_row(w.d, db_bits) / 1e9 / (scan_ms / args.steps * 1e-3),
            "traffic_GBps": (traffic / 1e9 / (scan_ms / max(launches, 1) * 1e-3)) if traffic else None,
        },
        "encode": {"db_ms": enc_ms,
                   "GBps": enc_bytes / 1e9 / (enc_ms * 1e-3),
                   "hbm_frac": enc_bytes / (enc_ms * 1e-3) / cm.HBM_BYTES_PER_S,
                   "measured_streaming_read_GBps": read_measured / 1e9,
                   "frac_of_measured_read": enc_bytes / (enc_ms * 1e-3) / read_measured,
                   "measured_same_traffic_no_arithmetic_GBps": None if mix_measured is None else mix_measured / 1e9,
                   "frac_of_same_traffic_no_arithmetic": None if mix_measured is None
                   else enc_bytes / (enc_ms * 1e-3) / mix_measured},
    }
    plain = args.refine < 0 and args.k_select < 0
    if plain and not args.no_few:
        for mq in (1, 4, 8):
            if mq <= w.m:
                out.setdefault("few_queries", []).append(
                    few_queries_leg(xbq, cm, w, Xdb, Xq, db, q, bits, db_bits, k, mq))
    # the cross-check scan (same integers from packed 4-bit dot products, d <= 256): what the
    # other formulation costs on this chip.  Reported beside the headline, never instead of it.
    if plain and not args.no_few and w.d <= 256 and not any(kv.startswith("kernel=") for kv in args.set):
        for kernel, label, note in ((1, "cross_check_dot8", "v_dot8_i32_i4 on nibble-packed codes"),
                                    (2, "cross_check_mfma", "v_mfma_i32_32x32x32_i8 on int8-decoded codes")):
            xbq.xbq_set_option("kernel", kernel)
            try:
                ws2 = torch.empty(xbq.xbq_search_workspace_bytes(w.n, w.m, w.d, bits, k), dtype=torch.uint8,
                                  device="cuda")
                idx2 = torch.empty_like(idx)
                sc2 = torch.empty_like(score)
                xbq.xbq_search_asym(db, w.n, db_bits, q, w.m, bits, w.d, k, workspace=ws2, idx=idx2, score=sc2)
                torch.cuda.synchronize()
                xbq.xbq_trace_enable(True)
                b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                b0.record()
                for _ in range(3):
                    xbq.xbq_search_asym(db, w.n, db_bits, q, w.m, bits, w.d, k, workspace=ws2, idx=idx2, score=sc2)
                b1.record()
                torch.cuda.synchronize()
                dms, _, _ = xbq.xbq_trace_read()
                xbq.xbq_trace_enable(False)
                out[label] = {
                    "search_ms": b0.elapsed_time(b1) / 3, "scan_ms": dms / 3,
                    "queries_per_s_search_only": w.m / (b0.elapsed_time(b1) / 3 * 1e-3),
                    "identical_to_xor_path": bool(torch.equal(idx2, idx) and torch.equal(sc2, score)),
                    "note": note + "; not the paper's XOR + popcount method"}
                del ws2, idx2, sc2
            finally:
                xbq.xbq_set_option("kernel", 0)
    if not args.no_recall:
        r, nq = recall_at_k(Xdb, Xq, idx, k)
        out["recall_at_k"] = {"value": r, "queries": nq, "against": "exact fp32 cosine (torch matmul + topk, in row slabs)"}
        out["recall_at_k"]["fp32_reference_max_abs_err_vs_f64"] = fp32_reference_error(Xdb, Xq)
        if not plain:
            out["recall_at_k"]["mean_candidates"] = float(ncand.float().mean())
            out["recall_at_k"]["max_candidates"] = int(ncand.max())
        else:
            out["recall_at_k"]["by_scale"] = recall_by_scale(xbq, wl, w, Xdb, Xq, bits, db_bits, k)
    del Xdb, Xq, db, q, ws, idx, score
    torch.cuda.empty_cache()
    # the same step on the other workloads (fewer steps each; the headline fields above stay C2)
    if plain and w.name == "C2" and not args.no_all and not args.queries and not args.set:
        out["all_workloads"] = [workload_summary(xbq, cm, wl, name, b, kk, st, 1) for name, b, kk, st in ALL_WORKLOADS]
    if plain and w.name == "C2" and not args.no_ordered and not args.no_all and not args.queries and not args.set:
        out["ordered_rows"] = ordered_rows_leg(xbq, wl)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, bits, db_bits, k, scale)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
