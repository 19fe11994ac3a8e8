"""GPU parity: every step of the HIP path against the CPU oracle on the same seeded inputs, through the
C ABI (paper_2403_05676_amd.binding -> libpiperag.so)."""
import os

import numpy as np
import pytest

import oracle
import parity
from workload import gen

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def P():
    import paper_2403_05676_amd as pkg
    pkg.load_library()
    return pkg


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make_problem(N, d, nlist, M, seed, ncomp=16, sigma=0.3, iters=4, nq=16, zipf=0.0):
    cfg = gen.WorkloadConfig(f"t{seed}", seed, ncomp, zipf, sigma, N, d, nlist, M, min(N, 20000), nq, 1, 1)
    x = gen.database(cfg)
    q = gen.queries(cfg, nq)
    S = min(N, 20000)
    ci = gen.draw_distinct_rows(S, nlist, seed)
    pi = [gen.draw_distinct_rows(S, 256, seed + 1 + m) for m in range(M)]
    coarse, pq = oracle.train(x[:S], nlist, M, ci, pi, iters=iters)
    return cfg, x, q, coarse, pq


def gpu_index_from_oracle(pkg, oidx: oracle.Index, **limits):
    """Library index holding exactly the oracle's lists (so that search parity does not depend on encoding ties)."""
    ix = pkg.Index.ivf_create(oidx.coarse, oidx.pq, oidx.ntotal, residual=oidx.residual, **limits)
    lists = np.repeat(np.arange(oidx.nlist, dtype=np.int32), np.diff(oidx.list_off))
    ix.ivf_add_encoded(dev(lists), dev(oidx.codes), dev(oidx.ids))
    ix.ivf_finalize()
    return ix


def run_search_parity(pkg, ix, oidx, q, nprobe, k):
    qd = dev(q)
    gl, gdist = ix.ivf_coarse(qd, nprobe)
    torch.cuda.synchronize()
    gl, gdist = gl.cpu().numpy(), gdist.cpu().numpy()
    ex_p = parity.check_probes(gl, gdist, q, oidx.coarse, nprobe)
    od, oi = ix.ivfpq_search(qd, nprobe, k)
    torch.cuda.synchronize()
    od, oi = od.cpu().numpy(), oi.cpu().numpy()
    ex_k, max_rel = parity.check_topk(od, oi, oidx, q, gl, k)
    scanned, nbytes = ix.search_stats()
    assert scanned == int(np.diff(oidx.list_off)[gl].sum())
    assert nbytes == scanned * oidx.M
    return ex_p, ex_k, max_rel


# ------------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def cfg0():
    cfg = gen.CONFIGS["cfg0"]
    x = gen.database(cfg)
    q = gen.queries(cfg)
    ci = gen.draw_distinct_rows(cfg.train_sample, cfg.nlist, cfg.seed)
    pi = [gen.draw_distinct_rows(cfg.train_sample, 256, cfg.seed + 1 + m) for m in range(cfg.M)]
    coarse, pq = oracle.train(x, cfg.nlist, cfg.M, ci, pi, iters=cfg.kmeans_iters)
    oidx = oracle.make_index(x, coarse, pq)
    return cfg, x, q, oidx


def test_cfg0_lut_and_coarse_taps(cfg0):
    cfg, x, q, oidx = cfg0
    pkg = P()
    ix = gpu_index_from_oracle(pkg, oidx)
    qd = dev(q)
    lut = ix.ivf_lut(qd)
    torch.cuda.synchronize()
    ref = oracle.lut(q, oidx.pq)
    assert np.all(parity.close(lut.cpu().numpy(), ref))
    gl, gd = ix.ivf_coarse(qd, cfg.nprobe)
    torch.cuda.synchronize()
    parity.check_probes(gl.cpu().numpy(), gd.cpu().numpy(), q, oidx.coarse, cfg.nprobe)
    gl, gd = ix.ivf_coarse(qd, cfg.nlist)            # full ordering of all lists
    torch.cuda.synchronize()
    parity.check_probes(gl.cpu().numpy(), gd.cpu().numpy(), q, oidx.coarse, cfg.nlist)


def test_cfg0_search_matches_oracle(cfg0):
    cfg, x, q, oidx = cfg0
    pkg = P()
    ix = gpu_index_from_oracle(pkg, oidx)
    ex_p, ex_k, max_rel = run_search_parity(pkg, ix, oidx, q, cfg.nprobe, cfg.k)
    print(f"cfg0: probe ties {ex_p}, top-k ties {ex_k}, max rel dist err {max_rel:.2e}")
    assert max_rel < 1e-4
    for nprobe, k in [(1, 1), (3, 100), (cfg.nlist, 10), (17, 128)]:
        run_search_parity(pkg, ix, oidx, q, nprobe, k)
    # single query, and a batch that is not a multiple of anything
    run_search_parity(pkg, ix, oidx, q[:1], 8, 10)
    run_search_parity(pkg, ix, oidx, q[:7], 8, 10)


def test_cfg0_gpu_encode_bit_exact_and_index_structure(cfg0):
    cfg, x, q, oidx = cfg0
    pkg = P()
    ix = pkg.Index.ivf_create(oidx.coarse, oidx.pq, cfg.N)
    xd = dev(x)
    gl, gc = ix.ivf_encode(xd)
    torch.cuda.synchronize()
    nl, nc = parity.check_encoding(gl.cpu().numpy(), gc.cpu().numpy(), x, oidx.coarse, oidx.pq)
    print(f"cfg0 encode: {nl} list and {nc} code-byte differences at ties, of {cfg.N} x {cfg.M}")
    assert nl <= cfg.N // 1000 and nc <= cfg.N * cfg.M // 1000
    # add in two uneven batches, then read every list back
    ix.ivf_add(xd[:40000])
    ix.ivf_add(xd[40000:])
    ix.ivf_finalize()
    assert ix.ivf_ntotal() == cfg.N
    lens = ix.ivf_list_lengths()
    assert lens.sum() == cfg.N
    glists = gl.cpu().numpy()
    gcodes = gc.cpu().numpy()
    seen = np.zeros(cfg.N, dtype=bool)
    for l in range(cfg.nlist):
        codes, ids = ix.ivf_get_list(l)
        assert len(ids) == lens[l]
        assert np.all(np.diff(ids) > 0)                       # order of addition = ascending id
        assert np.all(glists[ids] == l)                      # every vector sits in the list the encoder chose
        assert np.array_equal(codes, gcodes[ids])
        seen[ids] = True
    assert seen.all()
    # the oracle searching the GPU-built index gives what the GPU search gives
    off = np.zeros(cfg.nlist + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    parts = [ix.ivf_get_list(l) for l in range(cfg.nlist)]
    gidx = oracle.Index(oidx.coarse, oidx.pq, off, np.concatenate([p[0] for p in parts]),
                        np.concatenate([p[1] for p in parts]))
    run_search_parity(pkg, ix, gidx, q, cfg.nprobe, cfg.k)


def test_index_file_roundtrip(cfg0, tmp_path):
    cfg, x, q, oidx = cfg0
    pkg = P()
    path = str(tmp_path / "cfg0.ivfpq")
    oracle.write_index_file(oidx, path)
    ix = pkg.Index.ivf_load(path, max_nq=64, max_nprobe=64, max_k=32)
    assert (ix.d, ix.nlist, ix.M) == (cfg.d, cfg.nlist, cfg.M)
    run_search_parity(pkg, ix, oidx, q, cfg.nprobe, cfg.k)
    out = str(tmp_path / "saved.ivfpq")
    ix.ivf_save(out)
    assert open(out, "rb").read() == open(path, "rb").read()
    # truncated and corrupt files are rejected with an error code, not a crash
    raw = open(path, "rb").read()
    for bad in (raw[:40], raw[:len(raw) // 2], b"XXXXXXXX" + raw[8:]):
        p2 = str(tmp_path / "bad.ivfpq")
        open(p2, "wb").write(bad)
        with pytest.raises(pkg.PiperagError) as e:
            pkg.Index.ivf_load(p2)
        assert e.value.code == -4


# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,d,nlist,M,nprobe,k", [
    (5000, 32, 20, 1, 5, 10),        # one sub-quantiser
    (5000, 32, 20, 4, 20, 7),        # nprobe = nlist
    (3000, 24, 50, 8, 9, 100),       # ragged lists, k = 100
    (20000, 64, 33, 32, 6, 64),      # Mp = 32
    (20000, 96, 40, 24, 8, 33),      # M not a multiple of 16 (padded to 32)
    (9000, 96, 25, 48, 5, 20),       # Mp = 48
    (30000, 256, 64, 64, 12, 100),   # the M = 64 scan kernel
    (4000, 200, 16, 100, 4, 10),     # M = 100 (padded to 112), d not a multiple of 16
    (6000, 128, 30, 128, 7, 50),     # largest M
    (2500, 18, 12, 6, 3, 1000),      # k larger than most candidate sets, d % 4 != 0
])
def test_small_shapes_search_and_encode(N, d, nlist, M, nprobe, k):
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(N, d, nlist, M, seed=N + d + M, nq=9)
    oidx = oracle.make_index(x, coarse, pq)
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=16, max_nprobe=64, max_k=1024)
    run_search_parity(pkg, ix, oidx, q, nprobe, k)
    ix2 = pkg.Index.ivf_create(coarse, pq, N)
    gl, gc = ix2.ivf_encode(dev(x))
    torch.cuda.synchronize()
    parity.check_encoding(gl.cpu().numpy(), gc.cpu().numpy(), x, coarse, pq)


def test_empty_lists_few_candidates_and_given_probes():
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(300, 16, 64, 4, seed=5, nq=12)
    oidx = oracle.make_index(x[:90], coarse, pq)          # 90 vectors in 64 lists: some lists stay empty
    lens = np.diff(oidx.list_off)
    assert (lens == 0).any()
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=16, max_nprobe=64, max_k=64)
    run_search_parity(pkg, ix, oidx, q, 1, 40)       # most lists hold fewer than 40 vectors -> padding
    run_search_parity(pkg, ix, oidx, q, 64, 64)
    # probe lists chosen by the caller, including empty lists and skipped (-1) entries
    probes = np.full((len(q), 3), -1, dtype=np.int32)
    probes[:, 0] = int(np.argmin(lens))
    probes[:, 2] = np.arange(len(q)) % 64
    od, oi = ix.ivfpq_search_probes(dev(q), dev(probes), 20)
    torch.cuda.synchronize()
    parity.check_topk(od.cpu().numpy(), oi.cpu().numpy(), oidx, q, probes, 20)


def test_identity_codebook_is_exact_search():
    # dsub = 1, coordinates from a 256-value alphabet that is the codebook: IVF-PQ with nprobe = nlist
    # must return the exact nearest neighbours
    pkg = P()
    rng = np.random.default_rng(12)
    N, d, nlist = 4000, 16, 10
    alphabet = np.sort(rng.standard_normal(256)).astype(np.float32)
    x = alphabet[rng.integers(0, 256, size=(N, d))]
    q = rng.standard_normal((8, d)).astype(np.float32)
    pq = np.repeat(alphabet[None, :, None], d, 0)
    coarse = oracle.kmeans(x, nlist, gen.draw_distinct_rows(N, nlist, 1), 3)
    ix = pkg.Index.ivf_create(coarse, pq, N, max_nprobe=16, max_k=32)
    ix.ivf_add(dev(x))
    ix.ivf_finalize()
    od, oi = ix.ivfpq_search(dev(q), nlist, 20)
    torch.cuda.synchronize()
    bd, bi = oracle.brute_force_knn(x, q, 20)
    assert np.all(parity.close(od.cpu().numpy(), bd))
    got = oi.cpu().numpy()
    for a, b, dist in zip(got, bi, bd):
        clear = dist < dist[-1] * (1 - parity.RTOL)
        assert set(b[clear].tolist()) <= set(a.tolist())


def test_custom_ids_and_incremental_add():
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(4000, 32, 16, 8, seed=21, nq=5)
    ids = (np.arange(4000, dtype=np.int64) * 7919 + 10**12)
    oidx = oracle.make_index(x, coarse, pq, ids=ids)
    ix = pkg.Index.ivf_create(coarse, pq, 5000, max_k=16)
    xd, idd = dev(x), dev(ids)
    for a, b in [(0, 1), (1, 1000), (1000, 1000), (1000, 4000)]:
        ix.ivf_add(xd[a:b], idd[a:b])
    ix.ivf_finalize()
    od, oi = ix.ivfpq_search(dev(q), 4, 10)
    torch.cuda.synchronize()
    gl, _ = ix.ivf_coarse(dev(q), 4)
    torch.cuda.synchronize()
    parity.check_topk(od.cpu().numpy(), oi.cpu().numpy(), oidx, q, gl.cpu().numpy(), 10)


def test_argument_errors():
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(500, 16, 8, 4, seed=3, nq=4)
    ix = pkg.Index.ivf_create(coarse, pq, 500, max_nq=4, max_nprobe=4, max_k=8)
    qd = dev(q)
    with pytest.raises(pkg.PiperagError) as e:       # not finalized yet
        ix.ivfpq_search(qd, 2, 4)
    assert e.value.code == -1
    ix.ivf_add(dev(x))
    with pytest.raises(pkg.PiperagError) as e:       # beyond capacity
        ix.ivf_add(dev(x[:1]))
    assert e.value.code == -5
    ix.ivf_finalize()
    with pytest.raises(pkg.PiperagError) as e:
        ix.ivf_add(dev(x[:1]))
    assert e.value.code == -1
    for args, code in [((2, 9), -5), ((5, 4), -5), ((9, 4), -1), ((0, 4), -1), ((2, 0), -1)]:
        with pytest.raises(pkg.PiperagError) as e:
            ix.ivfpq_search(qd, *args)
        assert e.value.code == code, args
    with pytest.raises(pkg.PiperagError) as e:       # more queries than max_nq
        ix.ivfpq_search(torch.cat([qd, qd]), 2, 4)
    assert e.value.code == -5
    od, oi = ix.ivfpq_search(qd[:0], 2, 4)           # nq = 0 is a no-op
    assert od.shape == (0, 4)
    bad = dev(np.array([0, 99], dtype=np.int32))
    ix3 = pkg.Index.ivf_create(coarse, pq, 10)
    with pytest.raises(pkg.PiperagError) as e:       # list number out of range
        ix3.ivf_add_encoded(bad, dev(np.zeros((2, 4), np.uint8)))
    assert e.value.code == -1
    with pytest.raises(ValueError):
        pkg.Index.ivf_create(coarse, pq[:, :100], 10)


def test_results_are_deterministic(cfg0):
    cfg, x, q, oidx = cfg0
    pkg = P()
    ix = gpu_index_from_oracle(pkg, oidx)
    qd = dev(q)
    a = ix.ivfpq_search(qd, 16, 50)
    b = ix.ivfpq_search(qd, 16, 50)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_latency_profile_and_stage_times(cfg0):
    cfg, x, q, oidx = cfg0
    pkg = P()
    ix = gpu_index_from_oracle(pkg, oidx)
    qd = dev(q[:1])
    p50, fit = ix.latency_profile(qd, [1, 2, 4, 8, 16, 32, 64], 10, reps=5)
    assert np.all(p50 > 0) and fit[0] > 0              # positive intercept: the index scan (Section 3.1, O3)
    # the line is the least-squares fit of the returned medians (Section 3.2, S3: linear regression on nprobe)
    slope, intercept = np.polyfit(np.array([1, 2, 4, 8, 16, 32, 64], dtype=np.float64), p50.astype(np.float64), 1)
    assert abs(fit[1] - slope) <= 1e-4 * abs(slope) + 1e-7 and abs(fit[0] - intercept) <= 1e-4 * abs(intercept) + 1e-7
    ix.set_stage_timing(True)
    ix.ivfpq_search(qd, 8, 10)
    t = ix.stage_times()
    assert t.shape == (pkg.NSTAGES,) and np.all(t >= 0) and t.sum() > 0
    ix.set_stage_timing(False)


# ------------------------------------------------------------------------------------------------
def test_device_generator_is_bit_identical_to_numpy():
    from workload import gen_gpu
    for name, count in [("cfg0", 700), ("cfg1", 300)]:
        cfg = gen.CONFIGS[name]
        g = gen_gpu.DeviceGenerator(cfg)
        for row0 in (0, 12345, gen.QUERY_ROW0 + 3):
            a = g.rows(row0, count)
            torch.cuda.synchronize()
            assert np.array_equal(a.cpu().numpy(), gen.rows(cfg, row0, count))


def test_gpu_kmeans_follows_the_oracle():
    pkg = P()
    cfg = gen.CONFIGS["cfg0"].scaled(N=20000)
    x = gen.database(cfg)
    xd = dev(x)
    K = 40
    rows = gen.draw_distinct_rows(cfg.N, K, 77)
    # one iteration: same assignments (up to ties), means equal to fp32 rounding
    c1 = pkg.kmeans(xd, K, rows, 1).cpu().numpy()
    o1 = oracle.kmeans(x, K, rows, 1)
    np.testing.assert_allclose(c1, o1, rtol=2e-6, atol=2e-6)
    # zero iterations: the initial rows
    np.testing.assert_array_equal(pkg.kmeans(xd, K, rows, 0).cpu().numpy(), x[rows])
    # ten iterations: same trajectory of the objective
    c10, inert = pkg.kmeans(xd, K, rows, 10, return_inertia=True)
    o10, oin = oracle.kmeans(x, K, rows, 10, return_inertia=True)
    np.testing.assert_allclose(inert, oin, rtol=1e-3)
    assert np.all(np.diff(inert) <= 1e-6 * inert[0])
    # a column slice (one sub-quantiser's coordinates) with 256 centres
    rows2 = gen.draw_distinct_rows(cfg.N, 256, 78)
    s1 = pkg.kmeans(xd[:, 8:16], 256, rows2, 1).cpu().numpy()
    np.testing.assert_allclose(s1, oracle.kmeans(x[:, 8:16], 256, rows2, 1), rtol=2e-6, atol=2e-6)
    # deterministic
    assert torch.equal(pkg.kmeans(xd, K, rows, 3), pkg.kmeans(xd, K, rows, 3))


def test_long_lists_exercise_the_in_loop_candidate_pruning():
    # few long lists, many candidates per workgroup: the scan's candidate buffer fills up and is pruned
    # several times inside the scan loop (short lists never get there)
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(120000, 64, 4, 64, seed=99, nq=16, sigma=0.5, ncomp=4)
    oidx = oracle.make_index(x, coarse, pq)
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=16, max_nprobe=4, max_k=128)
    for k in (1, 100, 128):                     # ~29 blocks per workgroup, 16 per round: pruned in the first round
        run_search_parity(pkg, ix, oidx, q, 4, k)
    run_search_parity(pkg, ix, oidx, q[:1], 2, 100)
    # one query spread over more than a hundred workgroups: their keys are merged in two levels
    run_search_parity(pkg, ix, oidx, q[:1], 4, 100)
    run_search_parity(pkg, ix, oidx, q[:2], 4, 1)


def test_list_assignment_on_tight_clusters():
    # Clusters 12 times tighter than the benchmark's (sigma 0.02 against centres of norm ~ sqrt(768)): the distance
    # to the nearest centres is ~2,500 times smaller than |x||c|, which is what the rounding errors of the
    # expanded form |c|^2 - 2<x, c> are relative to.  A 16-significant-bit product would misplace vectors here by
    # far more than the tolerance; the shortlist product must be as accurate as fp32 and the direct-form
    # comparison of the two shortlisted centres must settle the rest.
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(32768, 768, 1024, 64, seed=31, ncomp=64, sigma=0.02, iters=2, nq=4)
    ix = pkg.Index.ivf_create(coarse, pq, cfg.N)
    gl, gc = ix.ivf_encode(dev(x))
    torch.cuda.synchronize()
    nl, nc = parity.check_encoding(gl.cpu().numpy(), gc.cpu().numpy(), x, coarse, pq)
    # how tight: the median ratio of |x||c| to the distance to the assigned centre
    ol, od = oracle.assign(x, coarse, return_dist=True)
    ratio = np.median(np.linalg.norm(x, axis=1) * np.linalg.norm(coarse[ol], axis=1) / np.maximum(od, 1e-30))
    print(f"tight clusters: |x||c| / distance = {ratio:.0f} (median); {nl} list and {nc} code-byte differences, all at ties")
    assert ratio > 1000
    assert nl <= 8                       # all excused as ties by check_encoding, and few


@pytest.mark.parametrize("N,d,nlist,M", [
    (6000, 72, 300, 9),              # two centre tiles, the second ragged; depth padded from 9 to 12 chunks of 8
    (5000, 100, 129, 25),            # one centre beyond a full tile; d not a multiple of 8
    (3000, 776, 513, 97),            # three tiles, one centre in the last; 97 chunks padded to 100
    (2000, 64, 1024, 8),             # the smallest depth the matrix-core path takes, whole tiles
])
def test_list_assignment_with_ragged_centre_tiles(N, d, nlist, M):
    # the matrix-core assignment walks the centres 256 at a time and the depth 16 at a time: places beyond the
    # last centre and beyond the last coordinate must not win or change a distance
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(N, d, nlist, M, seed=N + d + nlist, iters=2, nq=1)
    ix = pkg.Index.ivf_create(coarse, pq, N)
    gl, gc = ix.ivf_encode(dev(x))
    torch.cuda.synchronize()
    assert int(gl.min()) >= 0 and int(gl.max()) < nlist
    parity.check_encoding(gl.cpu().numpy(), gc.cpu().numpy(), x, coarse, pq)


def test_cross_workgroup_merge_is_repeatable():
    # One query spread over several hundred workgroups, merged in two levels (groups of workgroups, then the
    # groups): the keys cross workgroups through device-scope stores ordered by a counter.  200 identical searches
    # must each equal the first bit for bit, and the first must match the oracle; stops at the first mismatch.
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(400000, 64, 4, 64, seed=123, nq=4, sigma=0.5, ncomp=4)
    oidx = oracle.make_index(x, coarse, pq)
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=4, max_nprobe=4, max_k=128)
    for nq in (1, 3):
        qd = dev(q[:nq])
        run_search_parity(pkg, ix, oidx, q[:nq], 4, 100)
        d0, i0 = ix.ivfpq_search(qd, 4, 100)
        torch.cuda.synchronize()
        d0, i0 = d0.clone(), i0.clone()
        od = torch.empty_like(d0)
        oi = torch.empty_like(i0)
        for rep in range(200):
            od.fill_(-1.0); oi.fill_(-5)
            ix.ivfpq_search(qd, 4, 100, od, oi)
            torch.cuda.synchronize()
            assert torch.equal(od, d0) and torch.equal(oi, i0), f"repeat {rep} of the {nq}-query search differs from the first"


def test_many_vectors_with_identical_codes_tie_at_the_kth_distance():
    # a database of few distinct vectors, each repeated thousands of times: far more than k candidates share
    # every distance, so the bound on the k-th best distance alone never excludes them (ties are cut by slot)
    pkg = P()
    rng = np.random.default_rng(5)
    base = rng.standard_normal((48, 64)).astype(np.float32)
    x = base[rng.integers(0, 48, size=150000)]
    q = (base[:12] + 0.05 * rng.standard_normal((12, 64))).astype(np.float32)
    coarse = base[:4].copy()
    pq = np.ascontiguousarray(rng.standard_normal((8, 256, 8)).astype(np.float32))
    for m in range(8):
        pq[m, :48] = base[:, 8 * m:8 * m + 8]              # every distinct vector is encoded exactly
    oidx = oracle.make_index(x, coarse, pq)
    assert len(np.unique(oidx.codes, axis=0)) <= 48
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=16, max_nprobe=4, max_k=128)
    for k in (1, 100, 128):
        ex_p, ex_k, _ = run_search_parity(pkg, ix, oidx, q, 4, k)
        # which of the tied vectors are returned is decided by position, not id: most queries are "excused"
    od, oi = ix.ivfpq_search(dev(q), 4, 100)
    od2, oi2 = ix.ivfpq_search(dev(q), 4, 100)
    assert torch.equal(od, od2) and torch.equal(oi, oi2)   # and the choice is deterministic
    # results are ordered by (distance, id): inside a run of equal distances (here up to all 100 places) ids ascend
    dn, idn = od.cpu().numpy(), oi.cpu().numpy()
    assert (np.diff(dn, axis=1) >= 0).all()
    same = dn[:, 1:] == dn[:, :-1]
    assert same.sum() > 500 and (idn[:, 1:][same] > idn[:, :-1][same]).all()


def test_repeated_calls_replay_a_captured_graph_with_fresh_inputs(cfg0):
    # the third and later calls with the same buffers are graph replays: each must see the buffer's current
    # contents, with eager work and synchronisation in between, and agree with a plain call on other buffers
    cfg, x, q, oidx = cfg0
    pkg = P()
    ix = gpu_index_from_oracle(pkg, oidx)
    ix.set_graph_replay(True)
    rng = np.random.default_rng(11)
    qbuf = torch.empty((8, cfg.d), dtype=torch.float32, device="cuda")
    od = torch.empty((8, cfg.k), dtype=torch.float32, device="cuda")
    oi = torch.empty((8, cfg.k), dtype=torch.int64, device="cuda")
    for rep in range(6):
        sel = rng.integers(0, q.shape[0], size=8)
        qbuf.copy_(dev(q[sel]))
        ix.ivfpq_search(qbuf, cfg.nprobe, cfg.k, od, oi)
        junk = (torch.randn(1 << 16, device="cuda") * 2).sum()        # unrelated eager work between replays
        torch.cuda.synchronize()
        rd, ri = ix.ivfpq_search(dev(q[sel]), cfg.nprobe, cfg.k)      # fresh buffers: seen for the first time, plain path
        torch.cuda.synchronize()
        assert torch.equal(od, rd) and torch.equal(oi, ri), f"replay {rep} differs from the plain call"
        gl, _ = ix.ivf_coarse(qbuf, cfg.nprobe)
        torch.cuda.synchronize()
        parity.check_topk(od.cpu().numpy(), oi.cpu().numpy(), oidx, q[sel], gl.cpu().numpy(), cfg.k)
        assert float(junk) == float(junk)


def test_largest_nprobe_and_k():
    # the limits of a search call: nprobe = 1024 of 1100 short lists, k = 1024, one query and a small batch
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(40000, 32, 1100, 8, seed=321, nq=5, iters=2)
    oidx = oracle.make_index(x, coarse, pq)
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=8, max_nprobe=1024, max_k=1024)
    run_search_parity(pkg, ix, oidx, q, 1024, 1024)
    run_search_parity(pkg, ix, oidx, q[:1], 1024, 100)
    run_search_parity(pkg, ix, oidx, q, 1000, 1)


def test_scan_with_streaming_loads_gives_the_same_results(cfg0):
    # large indexes are scanned with non-temporal loads; forced here on a small one, against the oracle and
    # bit for bit against the ordinary loads
    pkg = P()
    cfg, x, q, oidx = cfg0
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=cfg.nq, max_nprobe=cfg.nlist, max_k=128)
    qd = dev(q)
    for nprobe, k in [(cfg.nprobe, cfg.k), (cfg.nlist, 100)]:
        ix.set_scan_streaming(0)
        d0, i0 = ix.ivfpq_search(qd, nprobe, k)
        ix.set_scan_streaming(1)
        run_search_parity(pkg, ix, oidx, q, nprobe, k)
        d1, i1 = ix.ivfpq_search(qd, nprobe, k)
        torch.cuda.synchronize()
        assert torch.equal(d0, d1) and torch.equal(i0, i1)
    ix.set_scan_streaming(-1)


def test_batches_larger_than_the_number_of_scan_workgroups():
    # 700 queries share 2048 scan workgroups; 2500 queries get one workgroup each
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(20000, 32, 64, 8, seed=99, nq=2500, iters=2)
    oidx = oracle.make_index(x, coarse, pq)
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=2500, max_nprobe=8, max_k=16)
    run_search_parity(pkg, ix, oidx, q[:700], 4, 10)
    run_search_parity(pkg, ix, oidx, q, 3, 5)


def test_seeded_random_shapes_match_the_oracle():
    # a seeded walk over code lengths, sub-vector lengths, list counts, probe counts, k and batch sizes, raw and
    # residual, with ordinary and streaming loads
    pkg = P()
    rng = np.random.default_rng(7)
    done = 0
    while done < 20:
        M = int(rng.choice([1, 2, 4, 8, 16, 24, 32, 48, 64, 96, 128]))
        d = M * int(rng.choice([1, 2, 3, 4, 6, 8, 12]))
        N = int(rng.integers(300, 40000))
        nlist = int(rng.integers(1, min(400, N // 2)))
        nprobe = int(rng.integers(1, nlist + 1))
        k = int(rng.choice([1, 2, 5, 10, 64, 100, 128, 129, 300, 1024]))
        nq = int(rng.choice([1, 2, 3, 5, 8, 17, 33, 64, 100]))
        residual = bool(rng.integers(0, 2))
        if d < 2 or d > 1024:
            continue
        if residual:
            cfg, x, q, coarse, pq = make_residual_problem(N, d, nlist, M, seed=1000 + done, nq=nq, iters=1)
            oidx = oracle.make_index_residual(x, coarse, pq)
        else:
            cfg, x, q, coarse, pq = make_problem(N, d, nlist, M, seed=1000 + done, nq=nq, iters=1)
            oidx = oracle.make_index(x, coarse, pq)
        ix = gpu_index_from_oracle(pkg, oidx, max_nq=nq, max_nprobe=nprobe, max_k=k)
        run_search_parity(pkg, ix, oidx, q, nprobe, k)
        ix.set_scan_streaming(1)
        run_search_parity(pkg, ix, oidx, q[:1], nprobe, k)
        ix.ivf_free()
        done += 1


def long_row_problem(adversarial):
    """40,000 centres (a row of coarse distances too long for the selection's LDS staging) and few vectors.
    adversarial: the centres close to the queries all sit at list numbers i with i mod 4096 < 512, so that
    bounding the row by minima over interleaved groups of lists keeps far too many of them."""
    rng = np.random.default_rng(77 + adversarial)
    nlist, d, M, N = 40000, 16, 4, 3000
    coarse = rng.normal(0.0, 1.0, (nlist, d)).astype(np.float32)
    if adversarial:
        far = (np.arange(nlist) % 4096) >= 512
        coarse[far] += np.float32(20.0)
    x = (coarse[rng.integers(0, nlist, N)] + rng.normal(0.0, 0.1, (N, d))).astype(np.float32)
    q = rng.normal(0.0, 1.0 if not adversarial else 0.3, (6, d)).astype(np.float32)
    pq = np.stack([oracle.kmeans(x[:, m * 4:(m + 1) * 4], 256, gen.draw_distinct_rows(N, 256, 5 + m), 2) for m in range(M)])
    return x, q, coarse, pq


@pytest.mark.parametrize("adversarial", [0, 1])
def test_probe_selection_over_rows_too_long_for_lds(adversarial):
    pkg = P()
    x, q, coarse, pq = long_row_problem(adversarial)
    oidx = oracle.make_index(x, coarse, pq)
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=8, max_nprobe=1024, max_k=16)
    for nq in (6, 1, 3):                   # matrix-core products finished by the selection; row-wise distances
        for nprobe in (1, 50, 1024):
            run_search_parity(pkg, ix, oidx, q[:nq], nprobe, 10)


def test_two_pass_build_gives_the_same_index_as_the_one_pass_build():
    pkg = P()
    cfg, x, q, coarse, pq = make_problem(50000, 64, 40, 16, seed=77, nq=6)
    xd = dev(x)
    ids = torch.arange(50000, dtype=torch.int64, device="cuda") * 3 + 7
    one = pkg.Index.ivf_create(coarse, pq, 50000)
    one.ivf_add(xd, ids)
    one.ivf_finalize()
    two = pkg.Index.ivf_create(coarse, pq, 50000)
    tiles = [(0, 13000), (13000, 13001), (13001, 40000), (40000, 50000)]       # ragged tiles, different in the two passes
    for a, b in tiles:
        two.ivf_count(xd[a:b])
    with pytest.raises(pkg.PiperagError):
        two.ivf_add(xd[:10])                                 # the two kinds of build do not mix
    with pytest.raises(pkg.PiperagError):
        two.ivf_place(xd[:10])                               # not before reserve
    two.ivf_reserve()
    with pytest.raises(pkg.PiperagError):
        two.ivf_finalize()                                   # nothing placed yet
    for a, b in [(0, 20000), (20000, 20064), (20064, 50000)]:
        two.ivf_place(xd[a:b], ids[a:b])
    with pytest.raises(pkg.PiperagError):
        two.ivf_place(xd[:1])                                # more than was counted
    two.ivf_finalize()
    assert np.array_equal(one.ivf_list_lengths(), two.ivf_list_lengths())
    for l in range(40):
        c1, i1 = one.ivf_get_list(l)
        c2, i2 = two.ivf_get_list(l)
        assert np.array_equal(c1, c2) and np.array_equal(i1, i2), f"list {l} differs"
    d1, r1 = one.ivfpq_search(dev(q), 8, 10)
    d2, r2 = two.ivfpq_search(dev(q), 8, 10)
    assert torch.equal(d1, d2) and torch.equal(r1, r2)
    # ids by position when none are given
    three = pkg.Index.ivf_create(coarse, pq, 1000)
    three.ivf_count(xd[:1000]); three.ivf_reserve(); three.ivf_place(xd[:600]); three.ivf_place(xd[600:1000]); three.ivf_finalize()
    got = np.sort(np.concatenate([three.ivf_get_list(l)[1] for l in range(40)]))
    assert np.array_equal(got, np.arange(1000))


# ---- residual variant -----------------------------------------------------------------------------
def make_residual_problem(N, d, nlist, M, seed, nq=9, sigma=0.3, ncomp=16, iters=4):
    cfg = gen.WorkloadConfig(f"r{seed}", seed, ncomp, 0.0, sigma, N, d, nlist, M, min(N, 20000), nq, 1, 1)
    x = gen.database(cfg)
    q = gen.queries(cfg, nq)
    S = min(N, 20000)
    ci = gen.draw_distinct_rows(S, nlist, seed)
    pi = [gen.draw_distinct_rows(S, 256, seed + 1 + m) for m in range(M)]
    coarse, pq = oracle.train_residual(x[:S], nlist, M, ci, pi, iters=iters)
    return cfg, x, q, coarse, pq


@pytest.mark.parametrize("N,d,nlist,M,nprobe,k", [
    (20000, 64, 33, 16, 6, 50),       # Mp = 16
    (30000, 256, 64, 64, 12, 100),    # the M = 64 scan kernel (two blocks in flight)
    (9000, 96, 25, 48, 25, 20),       # Mp = 48, nprobe = nlist
    (4000, 200, 16, 100, 4, 10),      # M = 100 (padded to 112)
    (3000, 18, 12, 6, 3, 300),        # d/M = 3: the VALU encoder; k beyond most candidate sets
])
def test_residual_index_search_and_encode(N, d, nlist, M, nprobe, k):
    pkg = P()
    cfg, x, q, coarse, pq = make_residual_problem(N, d, nlist, M, seed=N + d + M)
    oidx = oracle.make_index_residual(x, coarse, pq)
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=16, max_nprobe=64, max_k=512)
    run_search_parity(pkg, ix, oidx, q, nprobe, k)
    run_search_parity(pkg, ix, oidx, q[:1], nprobe, k)
    ix.set_scan_streaming(1)                    # the large-index variant of the scan
    run_search_parity(pkg, ix, oidx, q, nprobe, k)
    ix.set_scan_streaming(-1)
    # given probes (the constants of the lists are then computed by their own kernel), with a repeat and a gap
    probes = np.tile(np.arange(nprobe, dtype=np.int32), (q.shape[0], 1))
    probes[:, -1] = probes[:, 0]
    od, oi = ix.ivfpq_search_probes(dev(q), dev(probes), k)
    torch.cuda.synchronize()
    probes[:, -1] = -1
    parity.check_topk(od.cpu().numpy(), oi.cpu().numpy(), oidx, q, probes, k)
    # encoder, built both ways
    ix2 = pkg.Index.ivf_create(coarse, pq, N, residual=True)
    gl, gc = ix2.ivf_encode(dev(x))
    torch.cuda.synchronize()
    parity.check_encoding(gl.cpu().numpy(), gc.cpu().numpy(), x, coarse, pq, residual=True)
    ix2.ivf_add(dev(x)); ix2.ivf_finalize()
    ix3 = pkg.Index.ivf_create(coarse, pq, N, residual=True)
    ix3.ivf_count(dev(x)); ix3.ivf_reserve(); ix3.ivf_place(dev(x)); ix3.ivf_finalize()
    d2, i2 = ix2.ivfpq_search(dev(q), nprobe, min(k, 100))
    d3, i3 = ix3.ivfpq_search(dev(q), nprobe, min(k, 100))
    assert torch.equal(d2, d3) and torch.equal(i2, i3)


def test_residual_index_file_roundtrip(tmp_path):
    pkg = P()
    cfg, x, q, coarse, pq = make_residual_problem(6000, 32, 10, 8, seed=44)
    oidx = oracle.make_index_residual(x, coarse, pq)
    ix = gpu_index_from_oracle(pkg, oidx, max_nq=16, max_nprobe=16, max_k=64)
    path = str(tmp_path / "res.idx")
    ix.ivf_save(path)
    ix2 = pkg.Index.ivf_load(path, max_nq=16, max_nprobe=16, max_k=64)
    d1, i1 = ix.ivfpq_search(dev(q), 5, 20)
    d2, i2 = ix2.ivfpq_search(dev(q), 5, 20)
    assert torch.equal(d1, d2) and torch.equal(i1, i2)
    run_search_parity(pkg, ix2, oidx, q, 5, 20)
