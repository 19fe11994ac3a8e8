#!/usr/bin/env python3
"""Benchmark of the IVF-PQ search path on one MI355X.

A step = one call of piperag_ivfpq_search over one query batch (coarse quantiser, top-nprobe selection,
lookup tables, list scan with k-selection, merge), inputs resident in HBM.  The index is built on the GPU
from the seeded synthetic workload (generated on the device, trained with piperag_kmeans, encoded with
piperag_ivf_add); none of that is inside the timed region.  Prints one JSON line.

    python bench.py --gpus 1 --steps 200 --warmup 20 [--workload cfg1]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# The workload a plain `python bench.py` measures: the largest single-GPU configuration, one of the two the roofline
# target is stated on.  Its whole run takes about five and a half minutes, 4.8 of them the build of 1.07 G vectors
# (`--workload cfg3` is the other target configuration, 1.6 minutes).
DEFAULT_WORKLOAD = "cfg4"
PARITY_QUERIES = 32            # queries of the timed batch whose results are compared with the oracle
LATENCY_CALLS = 200            # single-query searches the p50 latency is taken over, each with another query


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_index(pkg, cfg, torch, tile_rows=262144, max_nq=None, max_nprobe=None, max_k=None, residual=False):
    """Generates the database on the device, trains and encodes on the GPU.  Returns (index, generator, info).
    residual: the codebooks are trained on, and the codes quantise, the vectors' residuals to their list centres."""
    from workload import gen, gen_gpu
    g = gen_gpu.DeviceGenerator(cfg)
    t0 = time.time()
    sample = g.database(0, cfg.train_sample)
    init_c = gen.draw_distinct_rows(cfg.train_sample, cfg.nlist, cfg.seed)
    coarse = pkg.kmeans(sample, cfg.nlist, init_c, cfg.kmeans_iters)
    torch.cuda.synchronize()
    log(f"[build] coarse centres trained, {time.time() - t0:.0f}s")
    pq = torch.empty((cfg.M, 256, cfg.dsub), dtype=torch.float32, device="cuda")
    if residual:                                        # the sample's residuals: lists from the library, subtraction by torch
        tmp = pkg.Index.ivf_create(coarse.cpu().numpy(), np.zeros((cfg.M, 256, cfg.dsub), dtype=np.float32), 1)
        for a in range(0, cfg.train_sample, tile_rows):
            lists, _ = tmp.ivf_encode(sample[a:a + tile_rows])
            sample[a:a + tile_rows] -= coarse[lists.long()]
        tmp.ivf_free()
    for m in range(cfg.M):
        init_m = gen.draw_distinct_rows(cfg.train_sample, 256, cfg.seed + 1 + m)
        pq[m] = pkg.kmeans(sample[:, m * cfg.dsub:(m + 1) * cfg.dsub], 256, init_m, cfg.kmeans_iters)
    torch.cuda.synchronize()
    t_train = time.time() - t0
    del sample
    ix = pkg.Index.ivf_create(coarse.cpu().numpy(), pq.cpu().numpy(), cfg.N, max_nq=max_nq or cfg.nq,
                              max_nprobe=max_nprobe or cfg.nprobe, max_k=max_k or cfg.k, residual=residual)
    t0 = time.time()
    buf = torch.empty((min(tile_rows, cfg.N), cfg.d), dtype=torch.float32, device="cuda")
    # a staging area of more than 32 GiB is not worth its memory: the database is generated twice instead
    two_pass = cfg.N * (cfg.M + 12) > (32 << 30)

    def sweep(step, what):
        t_log = time.time()
        for it, a in enumerate(range(0, cfg.N, tile_rows)):
            n = min(tile_rows, cfg.N - a)
            step(g.database(a, n, out=buf)[:n])
            if it % 4 == 3:                             # keep the launch queue short, so progress can be reported
                torch.cuda.synchronize()
                if time.time() - t_log > 20:
                    log(f"[build] {what} {a + n} of {cfg.N} vectors, {time.time() - t0:.0f}s")
                    t_log = time.time()
        torch.cuda.synchronize()

    if two_pass:
        sweep(ix.ivf_count, "assigned")
        ix.ivf_reserve()
        sweep(ix.ivf_place, "placed")
    else:
        sweep(ix.ivf_add, "encoded")
    t_encode = time.time() - t0
    del buf
    t0 = time.time()
    ix.ivf_finalize()
    t_final = time.time() - t0
    return ix, g, {"train_s": t_train, "encode_s": t_encode, "finalize_s": t_final,
                   "coarse": coarse, "pq": pq}


def host_copy(ix, coarse, pq, lists=None, residual=False):
    """The GPU-built index in the oracle's canonical form, read back list by list through the C ABI.  With
    `lists` given, only those lists are fetched and every other list is left empty (enough for an oracle
    search that probes only them)."""
    import oracle
    lens = ix.ivf_list_lengths()
    if lists is not None:
        keep = np.zeros(ix.nlist, dtype=bool)
        keep[np.asarray(lists, dtype=np.int64)] = True
        lens = np.where(keep, lens, 0)
    off = np.zeros(ix.nlist + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    codes = np.empty((int(off[-1]), ix.M), dtype=np.uint8)
    ids = np.empty(int(off[-1]), dtype=np.int64)
    for l in np.nonzero(lens)[0]:
        c, i = ix.ivf_get_list(int(l))
        codes[off[l]:off[l + 1]] = c
        ids[off[l]:off[l + 1]] = i
    return oracle.Index(coarse, pq, off, codes, ids, residual=residual)


def shorten(kernel_name):
    name = kernel_name.replace("(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0][:60]


def _grid_of(row):
    """Threads in the launch grid of one rocprofv3 CSV row (the column set differs between the two tables)."""
    if row.get("Grid_Size"):
        return int(row["Grid_Size"])
    if row.get("Grid_Size_X"):
        return int(row["Grid_Size_X"]) * int(row.get("Grid_Size_Y") or 1) * int(row.get("Grid_Size_Z") or 1)
    return 0


def duration_populations(v, gap=1.8):
    """Launches of one kernel and grid, split into populations of durations: the sorted durations are cut wherever
    one is more than `gap` times the one before it (the bench launches the scan on the timed batch, on smaller
    batches and on single queries with the same grid).  Returns [(tag, durations)], longest population first; one
    population has an empty tag."""
    vs = sorted(v)
    groups = [[vs[0]]]
    for a, b in zip(vs, vs[1:]):
        if b > gap * a:
            groups.append([])
        groups[-1].append(b)
    if len(groups) == 1:
        return [("", vs)]
    groups.reverse()
    return [(f" [population {i + 1} of {len(groups)}]", g) for i, g in enumerate(groups)]


def summarize_rocprof(root, command):
    """Short text summary of rocprofv3 --output-format csv results: per-kernel totals from the kernel trace and
    per-kernel means of every counter collected.  Launches of one kernel are listed per grid size, because the
    bench launches the search on the timed batch, on smaller batches and on a single query; where the grid is the
    same for all (the scan: spare workgroups exit at once), the launches are split into populations of
    durations (see duration_populations)."""
    import collections
    import csv
    lines = [f"command: {command}" if command else "command: (not given)"]
    for dirpath, _, files in os.walk(root):
        for f in sorted(files):
            path = os.path.join(dirpath, f)
            if f.endswith("kernel_trace.csv"):
                agg = collections.defaultdict(list)
                for r in csv.DictReader(open(path)):
                    agg[(r["Kernel_Name"], _grid_of(r))].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
                tot = sum(sum(v) for v in agg.values())
                lines.append(f"kernel trace ({f}): kernel, grid threads, calls, total us, average us, min us, max us, share")
                for (name, grid), v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
                    short = shorten(name)
                    for tag, g in duration_populations(v):
                        lines.append(f"  {short + tag:50s} {grid:9d} {len(g):6d} {sum(g):12.1f} {sum(g)/len(g):10.2f} {min(g):10.2f} "
                                     f"{max(g):10.2f} {100*sum(g)/tot:6.2f}%")
            if f.endswith("counter_collection.csv"):
                agg = collections.defaultdict(list)
                for r in csv.DictReader(open(path)):
                    agg[(shorten(r["Kernel_Name"]), _grid_of(r), r["Counter_Name"])].append(float(r["Counter_Value"]))
                lines.append(f"counters ({f}): kernel, grid threads, counter, dispatches, mean, min, max per dispatch")
                for (name, grid, ctr), v in sorted(agg.items()):
                    lines.append(f"  {name:44s} {grid:9d} {ctr:24s} {len(v):5d} {sum(v)/len(v):16.1f} {min(v):16.1f} {max(v):16.1f}")
    return "\n".join(lines)


def stored_traffic(workload):
    """(HBM bytes per scan launch, where the figure comes from) from the committed counter summary under profiles/,
    or (None, reason).  The figure is not measured by the run that prints it: hardware counters need a run under
    rocprofv3 --pmc of their own."""
    rel = os.path.join("profiles", f"adc_scan_traffic_{workload}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, f"no stored counter summary ({rel})"
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":")[1]), (f"stored: {rel} (FETCH_SIZE + WRITE_SIZE of rocprofv3 --pmc runs of this workload, "
                                               "each scaled by a plain copy kernel; not measured in this run)")
    return None, f"{rel} holds no traffic_bytes_per_launch line"


def exact_knn(g, cfg, torch, q, k, tile_rows=262144):
    """Harness only (not the library, not the oracle): exact squared-L2 top-k of the queries over the whole
    synthetic database, regenerated tile by tile and compared with torch matrix products."""
    nq = q.shape[0]
    best_d = torch.full((nq, k), float("inf"), device="cuda")
    best_i = torch.full((nq, k), -1, dtype=torch.int64, device="cuda")
    qn = (q * q).sum(1, keepdim=True)
    buf = torch.empty((min(tile_rows, cfg.N), cfg.d), dtype=torch.float32, device="cuda")
    for a in range(0, cfg.N, tile_rows):
        n = min(tile_rows, cfg.N - a)
        x = g.database(a, n, out=buf)[:n]
        dist = qn + (x * x).sum(1)[None, :] - 2.0 * (q @ x.T)
        d, i = torch.topk(dist, min(k, n), dim=1, largest=False)
        cd, ci = torch.cat([best_d, d], 1), torch.cat([best_i, i + a], 1)
        best_d, sel = torch.topk(cd, k, dim=1, largest=False)
        best_i = torch.gather(ci, 1, sel)
    return best_i


def nprobe_sweep(args, pkg, cfg, torch):
    """Latency against nprobe (single query and batch of 8, p50 of `reps` searches per point, with the linear
    fit latency = a + b * nprobe of the performance model of Section 3.2, S3) and recall@k of 1,000 queries against the
    exact neighbours, for nprobe = 1, 2, 4, ... up to the configuration's nprobe."""
    nprobes = [p for p in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024) if p <= cfg.nprobe]
    ix, g, info = build_index(pkg, cfg, torch, max_nq=64, max_nprobe=max(nprobes), residual=args.residual)
    nrec = 1000
    q = g.queries(nrec)
    p50_1, fit_1 = ix.latency_profile(q[:1].contiguous(), nprobes, cfg.k, reps=50)
    p50_8, fit_8 = ix.latency_profile(q[:8].contiguous(), nprobes, cfg.k, reps=50)
    log("[sweep] exact neighbours of the recall queries (torch harness)")
    truth = exact_knn(g, cfg, torch, q, cfg.k).cpu().numpy()
    rows = []
    for j, p in enumerate(nprobes):
        hits = 0
        for a in range(0, nrec, 64):
            _, oi = ix.ivfpq_search(q[a:a + 64].contiguous(), p, cfg.k)
            got = oi.cpu().numpy()
            hits += sum(len(np.intersect1d(got[r], truth[a + r])) for r in range(got.shape[0]))
        rows.append({"nprobe": p, "p50_ms_nq1": float(p50_1[j]), "p50_ms_nq8": float(p50_8[j]), "recall": hits / (nrec * cfg.k)})
        log(f"[sweep] nprobe {p}: {rows[-1]}")
    print(f"| nprobe | p50 ms (nq=1) | p50 ms (nq=8) | recall@{cfg.k} |")
    print("|---|---|---|---|")
    for r in rows:
        print(f"| {r['nprobe']} | {r['p50_ms_nq1']:.4f} | {r['p50_ms_nq8']:.4f} | {r['recall']:.4f} |")
    print(json.dumps({"workload": cfg.name, "k": cfg.k, "recall_queries": nrec, "reps": 50, "rows": rows,
                      "fit_nq1_ms": {"a": float(fit_1[0]), "b": float(fit_1[1])},
                      "fit_nq8_ms": {"a": float(fit_8[0]), "b": float(fit_8[1])}}), flush=True)


def overlap_demo(args, pkg, cfg, torch):
    """Performance-model-driven retrieval (Section 3.2, S3) hidden behind generation (S1) on one GPU.  The paper
    runs the retrieval on a server of its own; here the search gets a slice of the compute units (a stream with
    a compute-unit mask, piperag_stream_create_cu_slice) and the generation step the rest.  The latency line is
    fitted by piperag_latency_profile on the search's own stream (so it is the line of the slice), inverted by
    piperag_max_nprobe for the time a synthetic generation step takes, and the chosen search is run beside
    that step.  The generation step stands in for the decoder: per token one pass over a weight matrix plus a
    read of a key/value cache that grows with the sequence length (memory-bound, like decoding), so its
    duration T(C) grows linearly in the sequence length.  One table per size of the search's slice."""
    cap = min(1024, cfg.nlist)
    ix, g, info = build_index(pkg, cfg, torch, max_nq=1, max_nprobe=cap)
    q1 = g.queries(1)
    nprobes = sorted({int(p) for p in np.linspace(64, cap, 16)})      # the range the choice falls in, evenly spaced
    W = torch.randn((8192, 8192), dtype=torch.float32, device="cuda")             # 256 MiB of "weights"
    x = torch.randn(8192, dtype=torch.float32, device="cuda")
    kv = torch.randn((16384, 4096), dtype=torch.float32, device="cuda")           # 16 KiB of cache per position
    out_d = torch.empty((1, cfg.k), dtype=torch.float32, device="cuda")
    out_i = torch.empty((1, cfg.k), dtype=torch.int64, device="cuda")
    ncu = torch.cuda.get_device_properties(0).multi_processor_count

    def generate(L, tokens=2):
        for _ in range(tokens):
            torch.mv(W, x)
            kv[:L].sum(dim=0)

    def timed(sa, sb, fn_a, fn_b, reps=30):
        ts = []
        for r in range(reps + 5):
            torch.cuda.synchronize()
            e0, ea, eb = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            e0.record()
            if fn_a:
                with torch.cuda.stream(sa):
                    sa.wait_event(e0); fn_a(); ea.record()
            if fn_b:
                with torch.cuda.stream(sb):
                    sb.wait_event(e0); fn_b(); eb.record()
            torch.cuda.synchronize()
            ta = e0.elapsed_time(ea) if fn_a else 0.0
            tb = e0.elapsed_time(eb) if fn_b else 0.0
            if r >= 5:
                ts.append((ta, tb))
        return np.median(np.array(ts), axis=0)

    tables = []
    for slice_cus in args.overlap_cus:
        if slice_cus == 0:                               # no partition: both streams may use every compute unit
            sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        else:
            sb = pkg.stream_create_cu_slice(0, slice_cus)               # the search's slice ...
            sa = pkg.stream_create_cu_slice(slice_cus, ncu - slice_cus)  # ... and the rest for the generation step
        ix.set_compute_units(slice_cus)                  # launches sized to the slice (0: the whole device)
        # The latency line is fitted under the conditions it is used in (the paper fits it on the deployment
        # hardware): while generation steps run on the other stream and share the memory system with the search.
        torch.cuda.synchronize()
        with torch.cuda.stream(sa):
            for _ in range(1500):                        # about 0.4 s of queued generation work
                generate(8192)
        with torch.cuda.stream(sb):
            p50, fit = ix.latency_profile(q1, nprobes, cfg.k, reps=20)
        busy = not sa.query()                            # the generation stream was still busy when the profile ended
        torch.cuda.synchronize()
        log(f"[overlap] p50 ms by nprobe (generation beside it: {busy}): " + ", ".join(f"{p}: {t:.3f}" for p, t in zip(nprobes, p50)))
        assert busy, "the latency profile outlasted the queued generation steps"
        log(f"[overlap] search on {slice_cus or ncu} compute units: latency fit {fit[0]:.4f} ms + {fit[1] * 1e3:.3f} us * nprobe")
        # The line is the search's time on the GPU (events on its stream, the launches queued ahead).  A retrieval that
        # is waited for also pays for its four launches from the host; like the paper's term for network and query
        # encoding (Section 3.2, S3) that is a constant added to the line: measured once, as what a search at the
        # smallest nprobe of the profile takes beside a generation step, from the common start, beyond the line.
        small = lambda: ix.ivfpq_search(q1, nprobes[0], cfg.k, out_d, out_i)
        t_small = float(timed(sa, sb, lambda: generate(8192), small)[1])
        overhead = max(0.0, t_small - float(fit[0] + fit[1] * nprobes[0]))
        log(f"[overlap] a waited-for search at nprobe {nprobes[0]} beside a generation step: {t_small:.4f} ms -> overhead {overhead:.4f} ms")
        full = torch.cuda.Stream()
        rows = []
        for L in (1024, 4096, 8192, 16384):
            t_gen_full = float(timed(full, None, lambda: generate(L), None)[0])      # the step with the whole GPU to itself
            t_gen = float(timed(sa, None, lambda: generate(L), None)[0])             # ... and on its share of the compute units
            nprobe, fits, pred = pkg.max_nprobe(fit, t_gen, cap, overhead_ms=overhead)
            search = lambda: ix.ivfpq_search(q1, nprobe, cfg.k, out_d, out_i)
            t_ret = float(timed(None, sb, None, search)[1])
            both = timed(sa, sb, lambda: generate(L), search)
            rows.append({"seq_len": L, "t_gen_whole_gpu_ms": t_gen_full, "t_gen_ms": t_gen, "nprobe": nprobe, "fits": fits,
                         "predicted_ret_ms": pred, "t_ret_alone_ms": t_ret, "t_gen_overlapped_ms": float(both[0]),
                         "t_ret_overlapped_ms": float(both[1])})
            log(f"[overlap] {rows[-1]}")
        print(f"\nsearch on {slice_cus} of {ncu} compute units, generation on the other {ncu - slice_cus}" if slice_cus else
              f"\nno partition: both streams on all {ncu} compute units")
        print(f"latency line of the search: {fit[0]:.4f} ms + {fit[1] * 1e3:.3f} us x nprobe, plus {overhead:.4f} ms for a waited-for call")
        print("| sequence length | T(C), whole GPU, alone ms | T(C) on its share, alone ms | nprobe chosen | predicted retrieval ms | "
              "retrieval alone ms | T(C) with retrieval beside it ms | retrieval beside T(C) ms | hidden | T(C) slowed by |")
        print("|---|---|---|---|---|---|---|---|---|---|")
        for r in rows:
            hidden = r["t_ret_overlapped_ms"] <= r["t_gen_overlapped_ms"]
            slow = r["t_gen_overlapped_ms"] / r["t_gen_whole_gpu_ms"] - 1.0
            print(f"| {r['seq_len']} | {r['t_gen_whole_gpu_ms']:.3f} | {r['t_gen_ms']:.3f} | {r['nprobe']} | {r['predicted_ret_ms']:.3f} | "
                  f"{r['t_ret_alone_ms']:.3f} | {r['t_gen_overlapped_ms']:.3f} | {r['t_ret_overlapped_ms']:.3f} | "
                  f"{'yes' if hidden else 'no'} | {100 * slow:+.1f} % |")
        tables.append({"search_cus": slice_cus, "fit_ms": {"a": float(fit[0]), "b": float(fit[1])}, "overhead_ms": overhead, "rows": rows})
        if slice_cus:
            torch.cuda.synchronize()
            pkg.stream_destroy(sa)
            pkg.stream_destroy(sb)
    print(json.dumps({"workload": cfg.name, "tables": tables}), flush=True)


def read_reference(torch):
    """What a kernel that only reads reaches on this GPU, by launch shape: 8 GiB read with eight 16-byte loads in
    flight per lane, ordinary and non-temporal, from 256 to 4,096 workgroups of 256 threads (the scan runs 512 to
    2,048).  The reference the scan's fraction of the HBM peak is read against."""
    from workload import gen_gpu
    src = torch.empty(1 << 31, dtype=torch.float32, device="cuda").normal_()      # 8 GiB: far beyond every cache
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    nbytes = src.numel() * 4
    print("| workgroups | ordinary loads GB/s | of 8 TB/s | non-temporal loads GB/s | of 8 TB/s |")
    print("|---|---|---|---|---|")
    rows = []
    for wgs in (256, 512, 1024, 2048, 4096):
        rates = []
        for nt in (False, True):
            ts = []
            for r in range(7):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(); gen_gpu.stream_read(src, wgs, nt, sink); e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            rates.append(nbytes / (float(np.median(ts[2:])) * 1e-3) / 1e9)
        rows.append({"workgroups": wgs, "ordinary_GBps": rates[0], "nontemporal_GBps": rates[1]})
        print(f"| {wgs} | {rates[0]:.0f} | {rates[0] / HBM_PEAK_GBS:.3f} | {rates[1]:.0f} | {rates[1] / HBM_PEAK_GBS:.3f} |")
    print(json.dumps({"read_reference": rows, "bytes": nbytes}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=["cfg0", "cfg1", "cfg2", "cfg3", "cfg4", "paper"])
    ap.add_argument("--batches", type=int, default=8, help="different query batches the steps go round (default 8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-latency", action="store_true", help="skip the single-query latency loop and the scans at other batch sizes (counter runs: every scan launch is then the timed batch)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain 1 GiB copy kernel three times (reference for the HBM traffic counters)")
    ap.add_argument("--residual", action="store_true",
                    help="build a residual index (codes of the vectors' residuals to their list centres) instead of the raw-vector one")
    ap.add_argument("--nprobe-sweep", action="store_true",
                    help="instead of the bench line: latency and recall against nprobe on the chosen workload (meant for cfg2)")
    ap.add_argument("--overlap", action="store_true",
                    help="instead of the bench line: retrieval sized by the latency model, run beside a synthetic generation step")
    ap.add_argument("--overlap-cus", type=lambda t: [int(v) for v in t.split(",")], default=[0, 48, 64, 96],
                    help="with --overlap: compute units given to the search stream, one table per value (0 = no partition)")
    ap.add_argument("--read-reference", action="store_true",
                    help="instead of the bench line: the rate of a kernel that only reads, by launch shape (roofline reference)")
    ap.add_argument("--summarize", metavar="DIR", help="write a text summary of rocprofv3 CSV output found under DIR and exit")
    ap.add_argument("--command", default="", help="with --summarize: the command line that produced DIR")
    args = ap.parse_args()
    if args.summarize:
        print(summarize_rocprof(args.summarize, args.command))
        return
    if args.gpus != 1:
        print("bench.py measures one GPU: the library is single-GPU by design (no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2403_05676_amd as pkg
    from workload import gen
    pkg.load_library()                      # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = gen.CONFIGS[args.workload]
    if args.read_reference:
        read_reference(torch)
        return
    if args.nprobe_sweep:
        nprobe_sweep(args, pkg, cfg, torch)
        return
    if args.overlap:
        overlap_demo(args, pkg, cfg, torch)
        return
    log(f"[bench] building {cfg.name}: N={cfg.N} d={cfg.d} nlist={cfg.nlist} M={cfg.M}")
    ix, g, info = build_index(pkg, cfg, torch, max_nq=max(cfg.nq, 1), residual=args.residual)
    log(f"[bench] train {info['train_s']:.1f}s encode {info['encode_s']:.1f}s finalize {info['finalize_s']:.1f}s")
    # A step searches one batch of cfg.nq queries; the steps go round args.batches different batches (all resident
    # in HBM beforehand), so that no step finds the lists of its own queries left in the caches by the step before.
    nb = max(1, args.batches)
    q_all = g.queries(cfg.nq * nb)
    batches = [q_all[b * cfg.nq:(b + 1) * cfg.nq] for b in range(nb)]
    q = batches[0]                          # the batch checked against the oracle and timed on the CPU
    out_d = torch.empty((cfg.nq, cfg.k), dtype=torch.float32, device="cuda")
    out_i = torch.empty((cfg.nq, cfg.k), dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()

    # ---- whole-path throughput: W warm-up steps, then exactly K timed steps -------------------
    for s in range(args.warmup):
        ix.ivfpq_search(batches[s % nb], cfg.nprobe, cfg.k, out_d, out_i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        ix.ivfpq_search(batches[s % nb], cfg.nprobe, cfg.k, out_d, out_i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    qps = cfg.nq / (ms_per_step * 1e-3)

    # ---- per-stage durations (HIP events on the search stream) over the same K steps ----------
    ix.set_stage_timing(True)
    stage = np.zeros((args.steps, pkg.NSTAGES), dtype=np.float64)
    step_bytes = np.zeros(args.steps, dtype=np.float64)
    step_vecs = np.zeros(args.steps, dtype=np.float64)
    for s in range(args.steps):
        ix.ivfpq_search(batches[s % nb], cfg.nprobe, cfg.k, out_d, out_i)
        stage[s] = ix.stage_times()
        step_vecs[s], step_bytes[s] = ix.search_stats()       # counted on the device during this very search
    ix.set_stage_timing(False)
    stage_ms = stage.mean(axis=0)
    scan_ms = float(stage_ms[3])
    scanned_vecs, scanned_bytes = float(step_vecs.mean()), float(step_bytes.mean())
    achieved = step_bytes.sum() / (stage[:, 3].sum() * 1e-3) / 1e9
    # ---- the scan at other batch sizes of the same index (stage events, median of 10 calls each) ----
    by_nq = {}
    ix.set_stage_timing(True)
    for nq_x in sorted({1, 16, cfg.nq} - {cfg.nq}):
        if nq_x > cfg.nq or args.no_latency:
            continue
        fr = []
        for r in range(12):
            qs = q_all[(r * nq_x) % (q_all.shape[0] - nq_x + 1):][:nq_x].contiguous()
            ix.ivfpq_search(qs, cfg.nprobe, cfg.k, out_d[:nq_x], out_i[:nq_x])
            t_scan = float(ix.stage_times()[3])
            fr.append((ix.search_stats()[1] / (t_scan * 1e-3) / 1e9, t_scan))
        fr = fr[2:]
        by_nq[str(nq_x)] = {"scanned_code_GBps": float(np.median([f[0] for f in fr])),
                            "frac_of_hbm_peak": float(np.median([f[0] for f in fr])) / HBM_PEAK_GBS,
                            "scan_ms": float(np.median([f[1] for f in fr])), "calls": len(fr)}
    ix.set_stage_timing(False)
    ix.ivfpq_search(q, cfg.nprobe, cfg.k, out_d, out_i)      # the outputs checked below are those of the first batch
    torch.cuda.synchronize()

    # ---- single-query latency (host call -> stream synchronised), p50 --------------------------
    q1 = q[:1].contiguous()                 # the caller's query buffer, refilled with another query before every call
    lat = []
    # (its own number of calls, not the steps': single queries differ by a factor of ten in the vectors they scan)
    for r in range(0 if args.no_latency else args.warmup + LATENCY_CALLS):
        q1.copy_(q_all[r % q_all.shape[0]][None])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ix.ivfpq_search(q1, cfg.nprobe, cfg.k, out_d[:1], out_i[:1])
        torch.cuda.synchronize()
        if r >= args.warmup:
            lat.append((time.perf_counter() - t1) * 1e3)
    p50_1q = float(np.median(lat)) if lat else None

    traffic, traffic_src = stored_traffic(cfg.name)
    result = {
        "metric": "IVF-PQ queries/sec + scanned-code HBM GB/s at nprobe; p50 1-query latency",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={cfg.N} d={cfg.d} nlist={cfg.nlist} M={cfg.M}x8bit nq={cfg.nq} "
                               f"nprobe={cfg.nprobe} k={cfg.k} (Zipf Gaussian mixture, seed {cfg.seed})",
                   "nq": cfg.nq, "nprobe": cfg.nprobe, "k": cfg.k, "codes": "residual" if args.residual else "raw vector",
                   "query_batches": nb},
        "p50_1query_ms": p50_1q,
        "scanned_code_GBps": achieved,
        "scanned_vectors_per_batch": scanned_vecs,
        "stage_ms": {n: float(v) for n, v in zip(pkg.STAGE_NAMES, stage_ms)},
        "build_s": {k: round(info[k], 2) for k in ("train_s", "encode_s", "finalize_s")},
        "roofline": {"bound": "hbm", "kernel": "adc_scan_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
                     "bytes_per_launch": scanned_bytes, "avg_launch_ms": scan_ms,
                     "note": "the kernel's whole launch: table staging, scan, k-selection, merge of the query's partial "
                             "results, id gather and sort (there is no separate priming or merge kernel)"
                             + ("; this index's codes are about the size of the last-level cache, so part of the rate "
                                "is cache bandwidth, not HBM" if cfg.N * cfg.M <= (512 << 20) else "")},
        "scan_at_other_batch_sizes": by_nq,
    }

    if args.calibrate_copy:
        from workload import gen_gpu
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            gen_gpu.plain_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst

    # ---- the CPU oracle on this machine's host cores, same index, same queries --------------------
    if not args.no_cpu_baseline:
        import oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import parity
        coarse_h, pq_h = info["coarse"].cpu().numpy(), info["pq"].cpu().numpy()
        qh = q.cpu().numpy()
        # a bounded sample: the first ns queries of the first batch (the host copy holds the lists they probe)
        ns = min(cfg.nq, PARITY_QUERIES)
        qh = qh[:ns]
        gl0, _ = ix.ivf_coarse(q, cfg.nprobe)
        torch.cuda.synchronize()
        gl0 = gl0.cpu().numpy()[:ns]
        needed = np.union1d(gl0.ravel(), oracle.coarse_search(qh, coarse_h, cfg.nprobe)[0].ravel())
        hidx = host_copy(ix, coarse_h, pq_h, lists=needed, residual=args.residual)   # only the lists either side probes
        oracle.search(hidx, qh, cfg.nprobe, cfg.k)            # warm-up
        times = []
        t_budget = time.time()
        while len(times) < 3 or time.time() - t_budget < 12:      # about 12 s of CPU work
            t1 = time.perf_counter()
            od, oi, oprobes, oscanned = oracle.search(hidx, qh, cfg.nprobe, cfg.k)
            times.append(time.perf_counter() - t1)
        t_cpu = float(np.median(times))
        result["cpu_baseline"] = {"value": ns / t_cpu, "unit": "queries/s", "cores": oracle.num_threads(), "kind": "oracle",
                                  "sample": f"the first {ns} queries of the benchmark's first batch, median of {len(times)} runs "
                                            f"({sum(times):.1f} s of CPU work), search only",
                                  "scanned_code_GBps": float(oscanned.sum()) * cfg.M / t_cpu / 1e9}
        # sanity: the timed GPU configuration agrees with the oracle on these queries of this very batch
        parity.check_probes(gl0, None, qh, coarse_h, cfg.nprobe)
        ex, rel = parity.check_topk(out_d.cpu().numpy()[:ns], out_i.cpu().numpy()[:ns], hidx, qh, gl0, cfg.k)
        result["parity_vs_oracle"] = {"queries_checked": ns, "queries_with_tie_differences": ex, "max_rel_dist_err": rel}
    print(json.dumps(result, default=float), flush=True)


if __name__ == "__main__":
    main()
