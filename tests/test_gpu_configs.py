"""Benchmark configurations at full size, in the launch configuration bench.py times: the index is trained
and encoded on the GPU, slices of the encoder output are checked against the oracle, the structure of the
whole index is checked by invariants, and the oracle searches a host copy of the probed lists.

All five configurations run by default (cfg0 is covered by test_gpu_parity.py); cfg3 takes about two minutes and
cfg4 about six, almost all of it the build.  PIPERAG_SKIP=cfg3,cfg4 leaves configurations out (quick runs while
developing), PIPERAG_LARGE=paper adds the paper-shaped database (3 x 10^9 vectors, 230 GB of HBM).

Encoder check.  The plain oracle assigns a few hundred rows per second against 65,536 centres, so two slices are
checked: a small one by the plain oracle alone (lists and codes, `parity.check_encoding`), and the
1,048,576-row slice the large configurations name, whose codes go to the plain oracle and whose list numbers
go to `parity.check_lists_screened` (a library matrix product rules out far centres with a wide margin, the
oracle decides among the rest).  PIPERAG_SLICE_ROWS overrides the size of the large slice."""
import json
import os
import time

import numpy as np
import pytest

import oracle
import parity
from workload import gen

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

LARGE = set(filter(None, os.environ.get("PIPERAG_LARGE", "").split(",")))
SKIP = set(filter(None, os.environ.get("PIPERAG_SKIP", "").split(",")))
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def record(name, what):
    """Figures of the run, for the reader of the log and (when the folder exists) as a small JSON file."""
    print(f"[{name}] {json.dumps(what, default=float)}", flush=True)
    out = os.path.join(ROOT, "gpurun_out")
    if os.path.isdir(out):
        with open(os.path.join(out, f"config_check_{name}.jsonl"), "a") as f:
            f.write(json.dumps(what, default=float) + "\n")


def run_config(name, slice_rows, batches, max_check=64, plain_rows=4096, capsys=None):
    import paper_2403_05676_amd as pkg
    import bench
    pkg.load_library()
    cfg = gen.CONFIGS[name]
    t0 = time.time()
    max_nq = max(nq for nq, _ in batches)
    max_np = max(npr for _, npr in batches)
    # the build of the large configurations takes minutes: its progress lines (one every 20 s) go to the terminal even
    # when pytest captures output, so that whoever runs the suite sees that it is alive
    import contextlib
    with (capsys.disabled() if capsys is not None else contextlib.nullcontext()):
        ix, g, info = bench.build_index(pkg, cfg, torch, max_nq=max_nq, max_nprobe=max_np, max_k=cfg.k)
    print(f"\n[{name}] built in {time.time() - t0:.1f}s (train {info['train_s']:.1f} encode {info['encode_s']:.1f} "
          f"finalize {info['finalize_s']:.1f})", flush=True)
    coarse, pq = info["coarse"].cpu().numpy(), info["pq"].cpu().numpy()
    # ---- structure of the whole index
    lens = ix.ivf_list_lengths()
    assert ix.ivf_ntotal() == cfg.N and lens.sum() == cfg.N and lens.min() >= 0
    # ---- encoder against the plain oracle on a slice in the middle of the database
    row0 = (cfg.N // 2) // 64 * 64 + 17
    xs = g.database(row0, plain_rows)
    gl, gc = ix.ivf_encode(xs)
    torch.cuda.synchronize()
    xh = xs.cpu().numpy()
    gl_h, gc_h = gl.cpu().numpy(), gc.cpu().numpy()
    t1 = time.time()
    assert np.array_equal(xh, gen.database(cfg, row0, plain_rows))          # device generator == numpy generator
    nl, nc = parity.check_encoding(gl_h, gc_h, xh, coarse, pq)
    record(name, {"check": "encode, plain oracle", "rows": plain_rows, "first_row": row0, "list_differences_at_ties": nl,
                  "code_byte_differences_at_ties": nc, "seconds": round(time.time() - t1, 1)})
    assert nl <= max(2, plain_rows // 200) and nc <= plain_rows * cfg.M // 200
    # ---- and on the large slice: codes by the plain oracle, lists by the oracle among the centres a matrix product leaves
    slice_rows = int(os.environ.get("PIPERAG_SLICE_ROWS", slice_rows))
    row1 = (cfg.N // 3) // 64 * 64 + 5
    slice_rows = min(slice_rows, cfg.N - row1)
    t1 = time.time()
    xs = g.database(row1, slice_rows)
    gl, gc = ix.ivf_encode(xs)
    torch.cuda.synchronize()
    xh = xs.cpu().numpy()
    gl_h, gc_h = gl.cpu().numpy(), gc.cpu().numpy()
    assert np.array_equal(xh[:4096], gen.database(cfg, row1, 4096))
    nl, nfull = parity.check_lists_screened(gl_h, xs, xh, coarse)
    t2 = time.time()
    nc = parity.check_codes(gc_h, xh, pq)
    record(name, {"check": "encode, large slice (lists: oracle among screened centres; codes: plain oracle)", "rows": slice_rows,
                  "first_row": row1, "list_differences_at_ties": nl, "rows_given_to_the_plain_oracle": nfull,
                  "code_byte_differences_at_ties": nc, "seconds_lists": round(t2 - t1, 1), "seconds_codes": round(time.time() - t2, 1)})
    assert nl <= max(2, slice_rows // 200) and nc <= slice_rows * cfg.M // 200
    del xs
    # the slice's vectors sit in the lists the encoder chose, with those codes
    for l in np.unique(gl_h)[:8]:
        codes, ids = ix.ivf_get_list(int(l))
        assert np.all(np.diff(ids) > 0)
        sel = np.nonzero(gl_h == l)[0]
        pos = np.searchsorted(ids, row1 + sel)
        assert np.array_equal(ids[pos], row1 + sel) and np.array_equal(codes[pos], gc_h[sel])
    # ---- search against the oracle on a host copy of the probed lists
    for nq, nprobe in batches:
        q = g.queries(nq)
        qh = q.cpu().numpy()
        probes, pd = ix.ivf_coarse(q, nprobe)
        od, oi = ix.ivfpq_search(q, nprobe, cfg.k)
        torch.cuda.synchronize()
        scanned, nbytes = ix.search_stats()
        probes = probes.cpu().numpy()
        assert scanned == int(lens[probes].sum())
        # throughput of this launch configuration (HIP events per stage)
        ix.set_stage_timing(True)
        ts = []
        for _ in range(10):
            ix.ivfpq_search(q, nprobe, cfg.k)
            ts.append(ix.stage_times().copy())
        ix.set_stage_timing(False)
        t = np.median(np.array(ts), axis=0)
        print(f"[{name}] nq={nq} nprobe={nprobe}: scanned {scanned} vectors; stages us {np.round(t * 1e3, 1)}; scan "
              f"{nbytes / t[3] / 1e6:.0f} GB/s ({nbytes / t[3] / 1e6 / 80:.1f}% of HBM peak); {nq / t.sum() * 1e3:.0f} queries/s",
              flush=True)
        t1 = time.time()
        ex_p = parity.check_probes(probes, pd.cpu().numpy(), qh, coarse, nprobe)
        print(f"[{name}] probe sets checked ({ex_p} differ at ties), {time.time() - t1:.1f}s", flush=True)
        nchk = min(nq, max_check)                  # the oracle re-scans these queries' lists on the host
        t1 = time.time()
        hidx = bench.host_copy(ix, coarse, pq, lists=np.unique(probes[:nchk]))
        print(f"[{name}] host copy of {len(np.unique(probes[:nchk]))} probed lists ({hidx.ntotal} vectors), "
              f"{time.time() - t1:.1f}s", flush=True)
        odh, oih = od.cpu().numpy(), oi.cpu().numpy()
        ex_k, rel = 0, 0.0
        for a in range(0, nchk, 4):
            t1 = time.time()
            b = min(a + 4, nchk)
            e, r = parity.check_topk(odh[a:b], oih[a:b], hidx, qh[a:b], probes[a:b], cfg.k)
            ex_k, rel = ex_k + e, max(rel, r)
            print(f"[{name}] top-k of queries {a}..{min(a + 4, nchk) - 1} checked, {time.time() - t1:.1f}s", flush=True)
        record(name, {"check": "search", "nq": nq, "nprobe": nprobe, "k": cfg.k, "scanned_vectors": int(scanned),
                      "scan_us": round(float(t[3]) * 1e3, 1), "scan_GBps": round(nbytes / t[3] / 1e6), "queries_per_s": round(nq / t.sum() * 1e3),
                      "probe_sets_differing_at_ties": ex_p, "queries_checked": nchk, "queries_with_tie_differences": ex_k,
                      "max_rel_dist_err": rel})
        assert rel < 1e-4
    return ix


def skip_if_asked(name):
    if name in SKIP:
        pytest.skip(f"PIPERAG_SKIP names {name}")


def test_cfg1_full_size():
    skip_if_asked("cfg1")
    run_config("cfg1", 65536, [(64, 32), (1, 32)])


def test_cfg2_full_size():
    skip_if_asked("cfg2")
    run_config("cfg2", 65536, [(1, 1), (1, 32), (1, 256), (8, 1), (8, 64), (8, 256)])


def test_cfg3_full_size(capsys):
    skip_if_asked("cfg3")
    run_config("cfg3", 1 << 20, [(64, 64), (16, 64), (1, 64)], max_check=32, capsys=capsys)


def test_cfg4_full_size(capsys):
    skip_if_asked("cfg4")
    run_config("cfg4", 1 << 20, [(1, 128), (16, 128), (256, 128)], max_check=32, capsys=capsys)


@pytest.mark.skipif("paper" not in LARGE, reason="set PIPERAG_LARGE=paper (builds 3 G vectors in two passes, 230 GB of HBM)")
def test_paper_shaped_index(capsys):
    run_config("paper", 1 << 20, [(1, 64), (64, 64)], max_check=16, capsys=capsys)
