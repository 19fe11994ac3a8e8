"""Pins of the CPU oracle against facts that do not depend on the oracle itself:
exact brute force, the distance to the decoded vector, identity codebooks, a hand-worked table,
closed forms of k-means, library routines, and the monotonicity of the candidate set in nprobe."""
import os
import subprocess
import sys

import numpy as np
import pytest
from scipy.spatial.distance import cdist

import oracle
from workload import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_problem(N=2000, d=16, nlist=16, M=4, seed=11, ncomp=8):
    cfg = gen.WorkloadConfig("tiny", seed, ncomp, 0.0, 0.4, N, d, nlist, M, N, 20, 4, 10)
    x = gen.database(cfg)
    q = gen.queries(cfg)
    ci = gen.draw_distinct_rows(N, nlist, seed)
    pi = [gen.draw_distinct_rows(N, 256, seed + 1 + m) for m in range(M)]
    coarse, pq = oracle.train(x, nlist, M, ci, pi, iters=5)
    return cfg, x, q, coarse, pq


# ---------------------------------------------------------------- worked example (table, ADC, encode)
def read_golden():
    rows = {}
    codes = []
    with open(os.path.join(GOLDEN, "two_subquantizer_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            vals = [float(v) for v in vals]
            if key == "code":
                codes.append(vals)
            else:
                rows[key] = vals
    return rows, np.array(codes)


def test_worked_two_subquantizer_example():
    g, codes = read_golden()
    pq = np.array([np.array(g["P0"]).reshape(4, 2), np.array(g["P1"]).reshape(4, 2)], dtype=np.float32)
    q = np.array([g["q"]], dtype=np.float32)
    table = oracle.lut(q, pq)[0]
    assert table[0].tolist() == g["lut0"]
    assert table[1].tolist() == g["lut1"]
    # one list holding the six entries
    idx = oracle.Index(np.zeros((1, 4), np.float32), pq, np.array([0, 6], np.int64),
                       codes[:, :2].astype(np.uint8), np.arange(6, dtype=np.int64))
    dist, ids, _, scanned = oracle.search(idx, q, nprobe=1, k=6)
    assert scanned[0] == 6
    expect = codes[:, 2]
    assert sorted(dist[0].tolist()) == sorted(expect.tolist())
    assert ids[0, :3].tolist() == [int(v) for v in g["top3"][0::2]]
    assert dist[0, :3].tolist() == g["top3"][1::2]
    dec = oracle.decode(codes[5:6, :2].astype(np.uint8), pq)
    assert dec[0].tolist() == g["decoded5"]
    # encoding rule
    v = np.array([g["v"]], dtype=np.float32)
    _, vcode = oracle.encode(v, np.zeros((1, 4), np.float32), pq)
    assert vcode[0].tolist() == [int(c) for c in g["vcode"]]
    np.testing.assert_allclose(oracle.lut(v, pq)[0, 0], g["vsub0"], rtol=1e-6)
    np.testing.assert_allclose(oracle.lut(v, pq)[0, 1], g["vsub1"], rtol=1e-6)


# ---------------------------------------------------------------- brute force / library routines
def test_brute_force_knn_matches_library_distances():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((500, 7)).astype(np.float32)
    q = rng.standard_normal((9, 7)).astype(np.float32)
    dist, ids = oracle.brute_force_knn(x, q, 12)
    full = cdist(q.astype(np.float64), x.astype(np.float64), "sqeuclidean")
    order = np.argsort(full, axis=1, kind="stable")[:, :12]
    assert np.array_equal(ids, order)
    np.testing.assert_allclose(dist, np.take_along_axis(full, order, 1), rtol=1e-6)
    # more neighbours asked for than there are vectors: padded with (-1, +inf)
    dist, ids = oracle.brute_force_knn(x[:5], q, 8)
    assert np.all(ids[:, 5:] == -1) and np.all(np.isinf(dist[:, 5:]))


def test_assign_and_coarse_match_library_distances():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((300, 24)).astype(np.float32)
    c = rng.standard_normal((40, 24)).astype(np.float32)
    full = cdist(x.astype(np.float64), c.astype(np.float64), "sqeuclidean")
    idx, dist = oracle.assign(x, c, return_dist=True)
    assert np.array_equal(idx, np.argmin(full, axis=1))
    np.testing.assert_allclose(dist, full.min(axis=1), rtol=1e-6)
    probes, pd = oracle.coarse_search(x[:10], c, 7)
    assert np.array_equal(probes, np.argsort(full[:10], axis=1, kind="stable")[:, :7])
    np.testing.assert_allclose(pd, np.sort(full[:10], axis=1)[:, :7], rtol=1e-6)


def test_assign_ties_take_lowest_index():
    c = np.array([[1, 0], [0, 1], [1, 0], [-1, 0]], dtype=np.float32)   # centres 0 and 2 coincide
    x = np.array([[1, 0], [0, 0], [0.5, 0.5]], dtype=np.float32)
    assert oracle.assign(x, c).tolist() == [0, 0, 0]
    probes, _ = oracle.coarse_search(x[1:2], c, 4)
    assert probes[0].tolist() == [0, 1, 2, 3]


def test_assign_among_a_subset_of_the_centres():
    # pinned by SciPy's distances restricted to the listed centres; entries in any order, negative ones skipped,
    # equal distances to the lower centre number; with every centre listed it is the full assignment
    rng = np.random.default_rng(11)
    x = rng.standard_normal((200, 24)).astype(np.float32)
    c = rng.standard_normal((50, 24)).astype(np.float32)
    full = cdist(x.astype(np.float64), c.astype(np.float64), "sqeuclidean")
    cand = np.stack([rng.permutation(50)[:6] for _ in range(200)]).astype(np.int32)
    cand[::3, 2] = -1
    idx, dist = oracle.assign_among(x, c, cand, return_dist=True)
    for i in range(200):
        valid = cand[i][cand[i] >= 0]
        want = valid[np.argmin(full[i, valid])]
        assert idx[i] == want
        assert abs(dist[i] - full[i, want]) <= 1e-6 * full[i, want]
    everything = np.stack([rng.permutation(50) for _ in range(200)]).astype(np.int32)
    assert np.array_equal(oracle.assign_among(x, c, everything), oracle.assign(x, c))
    # ties: centres 0 and 2 coincide; listed as (2, 0) the answer is still 0
    c2 = np.array([[1, 0], [0, 1], [1, 0], [-1, 0]], dtype=np.float32)
    x2 = np.array([[1, 0], [0.5, 0.5]], dtype=np.float32)
    assert oracle.assign_among(x2, c2, np.array([[2, 0], [2, 1]], dtype=np.int32)).tolist() == [0, 1]
    # the codes-only entry equals the code part of the full encoding
    pq = rng.standard_normal((4, 256, 6)).astype(np.float32)
    assert np.array_equal(oracle.encode_codes(x, pq), oracle.encode(x, c, pq)[1])


def test_adc_equals_distance_to_decoded_vector():
    cfg, x, q, coarse, pq = small_problem()
    idx = oracle.make_index(x, coarse, pq)
    dist, ids, probes, scanned = oracle.search(idx, q, nprobe=cfg.nlist, k=25)
    assert np.all(scanned == cfg.N)
    dec = oracle.decode(idx.codes, pq)                       # rows in list order
    full = cdist(q.astype(np.float64), dec.astype(np.float64), "sqeuclidean")
    pos = np.empty(cfg.N, dtype=np.int64)
    pos[idx.ids] = np.arange(cfg.N)
    got = np.take_along_axis(full, pos[ids], 1)
    np.testing.assert_allclose(dist, got, rtol=1e-6)
    # and they are the 25 smallest such distances
    np.testing.assert_allclose(dist, np.sort(full, axis=1)[:, :25], rtol=1e-6)
    # every vector sits in the list of its nearest centre, and codes pick the nearest sub-centre
    assert np.array_equal(np.repeat(np.arange(cfg.nlist), np.diff(idx.list_off)),
                          np.argmin(cdist(x[idx.ids].astype(np.float64), coarse.astype(np.float64), "sqeuclidean"), 1))
    m = 2
    sub = x[idx.ids][:, m * cfg.dsub:(m + 1) * cfg.dsub].astype(np.float64)
    assert np.array_equal(idx.codes[:, m], np.argmin(cdist(sub, pq[m].astype(np.float64), "sqeuclidean"), 1))


# ---------------------------------------------------------------- identity codebooks => exact search
def test_identity_codebook_small_database_is_exact_search():
    # every database vector is its own code: P[m][j] = m-th slice of vector j  (N <= 256)
    rng = np.random.default_rng(3)
    N, d, M, nlist = 200, 12, 4, 8
    x = rng.standard_normal((N, d)).astype(np.float32)
    q = rng.standard_normal((15, d)).astype(np.float32)
    pq = np.full((M, 256, d // M), 1e3, dtype=np.float32)      # unused centres far away
    for m in range(M):
        pq[m, :N] = x[:, m * 3:(m + 1) * 3]
    coarse = oracle.kmeans(x, nlist, gen.draw_distinct_rows(N, nlist, 5), 4)
    idx = oracle.make_index(x, coarse, pq)
    assert np.array_equal(idx.codes, np.repeat(idx.ids[:, None], M, 1).astype(np.uint8))
    dist, ids, _, _ = oracle.search(idx, q, nprobe=nlist, k=10)
    bd, bi = oracle.brute_force_knn(x, q, 10)
    assert np.array_equal(ids, bi)
    np.testing.assert_allclose(dist, bd, rtol=1e-6)


def test_identity_codebook_scalar_alphabet_is_exact_search():
    # dsub = 1 and every coordinate drawn from a 256-value alphabet which is the codebook (any N)
    rng = np.random.default_rng(4)
    N, d, nlist = 3000, 8, 12
    alphabet = np.sort(rng.standard_normal(256)).astype(np.float32)
    x = alphabet[rng.integers(0, 256, size=(N, d))]
    q = rng.standard_normal((10, d)).astype(np.float32)
    pq = np.repeat(alphabet[None, :, None], d, 0)              # [M=d, 256, 1]
    coarse = oracle.kmeans(x, nlist, gen.draw_distinct_rows(N, nlist, 6), 4)
    idx = oracle.make_index(x, coarse, pq)
    np.testing.assert_array_equal(oracle.decode(idx.codes, pq), x[idx.ids])
    dist, ids, _, _ = oracle.search(idx, q, nprobe=nlist, k=20)
    bd, bi = oracle.brute_force_knn(x, q, 20)
    np.testing.assert_allclose(dist, bd, rtol=1e-6)
    for a, b, da in zip(ids, bi, dist):                        # ids equal wherever distances are distinct
        distinct = np.concatenate([[True], np.diff(da) > 0]) & np.concatenate([np.diff(da) > 0, [False]])
        assert np.array_equal(a[distinct], b[distinct])
        assert set(a[da < da[-1]]) == set(b[da < da[-1]])


# ---------------------------------------------------------------- monotonicity in nprobe
def test_candidate_set_and_recall_monotone_in_nprobe():
    cfg, x, q, coarse, pq = small_problem(N=4000, nlist=32)
    idx = oracle.make_index(x, coarse, pq)
    k = 10
    exhaustive = oracle.search(idx, q, cfg.nlist, k)[1]
    exact = oracle.brute_force_knn(x, q, k)[1]
    prev_probes = None
    prev_kth = np.full(len(q), np.inf)
    prev_scanned = np.zeros(len(q))
    prev_rec = -1.0
    recalls_exact = []
    for p in [1, 2, 3, 4, 8, 16, 32]:
        dist, ids, probes, scanned = oracle.search(idx, q, p, k)
        if prev_probes is not None:                            # probe lists are prefixes of each other
            assert np.array_equal(probes[:, :prev_probes.shape[1]], prev_probes)
        assert np.all(scanned >= prev_scanned)
        assert np.all(scanned == [np.diff(idx.list_off)[pr].sum() for pr in probes])
        kth = dist[:, -1]
        assert np.all(kth <= prev_kth)
        rec = oracle.recall_at_k(ids, exhaustive)
        assert rec >= prev_rec
        recalls_exact.append(oracle.recall_at_k(ids, exact))
        prev_probes, prev_kth, prev_scanned, prev_rec = probes, kth, scanned, rec
    assert prev_rec == 1.0                                      # nprobe = nlist scans everything
    assert np.all(prev_scanned == cfg.N)
    assert recalls_exact[-1] >= recalls_exact[0]                # plateau is above the start (Section 3.1, O3)
    assert 0.0 < recalls_exact[-1] <= 1.0


def test_search_with_probes_pads_and_skips():
    cfg, x, q, coarse, pq = small_problem(N=300, nlist=64)
    idx = oracle.make_index(x, coarse, pq)
    probes = np.full((len(q), 3), -1, dtype=np.int32)
    empty = int(np.argmin(np.diff(idx.list_off)))
    probes[:, 0] = empty
    dist, ids, scanned = oracle.search_with_probes(idx, q, probes, 5)
    n = int(np.diff(idx.list_off)[empty])
    assert np.all(scanned == n) and n < 5
    assert np.all(ids[:, n:] == -1) and np.all(np.isinf(dist[:, n:]))


# ---------------------------------------------------------------- k-means closed forms
def test_kmeans_closed_forms():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((257, 5)).astype(np.float32)
    c = oracle.kmeans(x, 1, np.array([3]), 3)
    np.testing.assert_array_equal(c[0], x.astype(np.float64).mean(0).astype(np.float32))
    rows = gen.draw_distinct_rows(257, 257, 1)
    c, inertia = oracle.kmeans(x, 257, rows, 2, return_inertia=True)
    np.testing.assert_array_equal(c, x[rows])
    assert np.all(inertia == 0.0)
    c, inertia = oracle.kmeans(x, 9, gen.draw_distinct_rows(257, 9, 2), 10, return_inertia=True)
    assert np.all(np.diff(inertia) <= 1e-9 * inertia[0])
    # a centre that never gets a row keeps its value
    y = np.array([[0, 0], [0, 0], [5, 5]], dtype=np.float32)
    c = oracle.kmeans(y, 3, np.array([0, 1, 2]), 3)
    np.testing.assert_array_equal(c, [[0, 0], [0, 0], [5, 5]])
    # two well separated blobs converge to the blob means
    a = rng.standard_normal((50, 3)).astype(np.float32) * 0.1
    b = rng.standard_normal((60, 3)).astype(np.float32) * 0.1 + 10
    z = np.concatenate([a, b])
    c = oracle.kmeans(z, 2, np.array([0, 50]), 5)
    np.testing.assert_allclose(c[0], a.astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(c[1], b.astype(np.float64).mean(0), rtol=1e-6)


def test_kmeans_strided_slice_equals_copy():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((400, 12)).astype(np.float32)
    rows = gen.draw_distinct_rows(400, 16, 9)
    a = oracle.kmeans(x[:, 4:8], 16, rows, 4)
    b = oracle.kmeans(np.ascontiguousarray(x[:, 4:8]), 16, rows, 4)
    np.testing.assert_array_equal(a, b)


def test_kmeans_independent_of_thread_count():
    code = ("import numpy as np, oracle, hashlib; from workload import gen;"
            "cfg=gen.CONFIGS['cfg0'].scaled(N=4096); x=gen.database(cfg);"
            "c=oracle.kmeans(x,32,gen.draw_distinct_rows(4096,32,0),4);"
            "l,co=oracle.encode(x[:512],c,np.repeat(c[:,:8][None,:,:],16,0).repeat(8,1));"
            "print(hashlib.sha1(c.tobytes()+l.tobytes()+co.tobytes()).hexdigest())")
    root = os.path.dirname(os.path.dirname(__file__))
    outs = []
    for nt in ("1", "3"):
        env = dict(os.environ, OMP_NUM_THREADS=nt, PYTHONPATH=root)
        outs.append(subprocess.check_output([sys.executable, "-c", code], env=env, cwd=root).strip())
    assert outs[0] == outs[1]


# ---------------------------------------------------------------- structure of the built index
def test_index_structure_invariants():
    cfg, x, q, coarse, pq = small_problem(N=1500, nlist=24)
    idx = oracle.make_index(x, coarse, pq)
    assert idx.list_off[0] == 0 and idx.list_off[-1] == cfg.N
    assert np.all(np.diff(idx.list_off) >= 0)
    assert np.array_equal(np.sort(idx.ids), np.arange(cfg.N))
    for l in range(cfg.nlist):
        seg = idx.ids[idx.list_off[l]:idx.list_off[l + 1]]
        assert np.all(np.diff(seg) > 0)


def test_index_file_layout(tmp_path):
    cfg, x, q, coarse, pq = small_problem(N=300, nlist=4)
    idx = oracle.make_index(x, coarse, pq)
    path = tmp_path / "a.ivfpq"
    oracle.write_index_file(idx, str(path))
    raw = path.read_bytes()
    assert raw[:8] == b"PRAGIVF1"
    assert len(raw) == 64 + 4 * (4 * 16 + 4 * 256 * 4) + 8 * 4 + 300 * 4 + 8 * 300


def test_scan_with_probes_lists_every_candidate_once_and_its_k_best_are_the_search_result():
    """The all-candidates tap and the search share one scan: sorting the tap's output by (distance, id) and
    cutting at k must reproduce search_with_probes, and the candidate count is the sum of the list lengths."""
    rng = np.random.default_rng(77)
    x = rng.standard_normal((3000, 32)).astype(np.float32)
    coarse = x[:16].copy()                                     # any centres and codebooks do for this property
    pq = rng.standard_normal((8, 256, 4)).astype(np.float32)
    index = oracle.make_index(x, coarse, pq)
    q = rng.standard_normal((5, 32)).astype(np.float32)
    probes, _ = oracle.coarse_search(q, index.coarse, 4)
    probes[2, 1] = -1                                          # a skipped probe
    od, oi, scanned = oracle.search_with_probes(index, q, probes, 20)
    lens = np.diff(index.list_off)
    for qi in range(5):
        ad, ai = oracle.scan_with_probes(index, q[qi], probes[qi])
        assert len(ad) == scanned[qi] == lens[probes[qi][probes[qi] >= 0]].sum()
        assert len(set(ai.tolist())) == len(ai)
        order = np.lexsort((ai, ad))[:20]
        assert np.array_equal(ai[order], oi[qi]) and np.array_equal(ad[order], od[qi])


# ---- residual variant -----------------------------------------------------------------------------
def _residual_problem(seed=3, n=4000, d=24, nlist=12, M=6):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((nlist, d)).astype(np.float32) * 3
    x = (centres[rng.integers(0, nlist, n)] + 0.4 * rng.standard_normal((n, d))).astype(np.float32)
    ci = rng.choice(n, nlist, replace=False)
    pi = [rng.choice(n, 256, replace=False) for _ in range(M)]
    coarse, pq = oracle.train_residual(x, nlist, M, ci, pi, iters=4)
    return rng, x, coarse, pq


def test_residual_distance_is_the_distance_to_the_reconstructed_vector():
    """dist(q, x) of the residual variant must equal |q - (c_l + decode(code))|^2, the identity of its definition;
    a wrong sign of the centre, a residual taken to the wrong list or a table built on q instead of q - c fails it."""
    rng, x, coarse, pq = _residual_problem()
    index = oracle.make_index_residual(x, coarse, pq)
    assert index.residual
    q = rng.standard_normal((5, x.shape[1])).astype(np.float32) * 2
    probes, _ = oracle.coarse_search(q, coarse, 4)
    recon = oracle.decode(index.codes, pq).astype(np.float64)
    list_of = np.repeat(np.arange(index.nlist), np.diff(index.list_off))
    recon += coarse[list_of].astype(np.float64)
    for qi in range(5):
        ad, ai = oracle.scan_residual_with_probes(index, q[qi], probes[qi])
        pos = {int(i): p for p, i in enumerate(index.ids)}
        for dist, vid in list(zip(ad, ai))[::37]:
            p = pos[int(vid)]
            want = ((q[qi].astype(np.float64) - recon[p]) ** 2).sum()
            assert abs(dist - want) <= 1e-4 * want + 1e-5


def test_residual_variant_with_zero_centres_is_the_raw_variant():
    """With every coarse centre at the origin the residual is the vector itself: encoding and search must coincide
    with the raw-vector functions (which have their own pins)."""
    rng = np.random.default_rng(8)
    x = rng.standard_normal((1500, 16)).astype(np.float32)
    pq = rng.standard_normal((4, 256, 4)).astype(np.float32)
    coarse = np.zeros((3, 16), dtype=np.float32)
    l_r, c_r = oracle.encode_residual(x, coarse, pq)
    l_0, c_0 = oracle.encode(x, coarse, pq)
    assert np.array_equal(l_r, l_0) and np.array_equal(c_r, c_0)
    idx_r = oracle.make_index_residual(x, coarse, pq)
    idx_0 = oracle.make_index(x, coarse, pq)
    q = rng.standard_normal((4, 16)).astype(np.float32)
    probes = np.zeros((4, 1), dtype=np.int32)
    dr, ir, _ = oracle.search_residual_with_probes(idx_r, q, probes, 20)
    d0, i0, _ = oracle.search_with_probes(idx_0, q, probes, 20)
    assert np.array_equal(ir, i0) and np.array_equal(dr, d0)


def test_residual_codes_beat_raw_codes_on_clustered_data_and_exhaustive_probing_finds_the_best_reconstruction():
    """Residual codes spend their bits on the spread inside a list: on clustered data the reconstruction error is
    smaller than with raw-vector codes of the same size.  With nprobe = nlist the top-1 of the residual search is
    the vector whose reconstruction is closest to the query (brute force over reconstructions)."""
    rng, x, coarse, pq_res = _residual_problem(seed=5)
    n, d = x.shape
    ci = rng.choice(n, 12, replace=False)
    pi = [rng.choice(n, 256, replace=False) for _ in range(6)]
    _, pq_raw = oracle.train(x, 12, 6, ci, pi, iters=4)
    idx_res = oracle.make_index_residual(x, coarse, pq_res)
    idx_raw = oracle.make_index(x, coarse, pq_raw)
    list_of = np.repeat(np.arange(12), np.diff(idx_res.list_off))
    rec_res = oracle.decode(idx_res.codes, pq_res) + coarse[list_of]
    rec_raw = oracle.decode(idx_raw.codes, pq_raw)
    err_res = ((x[idx_res.ids] - rec_res) ** 2).sum(1).mean()
    err_raw = ((x[idx_raw.ids] - rec_raw) ** 2).sum(1).mean()
    assert err_res < err_raw
    q = x[rng.integers(0, n, 6)] + 0.1 * rng.standard_normal((6, d)).astype(np.float32)
    probes = np.tile(np.arange(12, dtype=np.int32), (6, 1))
    dr, ir, _ = oracle.search_residual_with_probes(idx_res, q, probes, 1)
    bd, bi = oracle.brute_force_knn(rec_res, q, 1)
    assert np.array_equal(idx_res.ids[bi[:, 0]], ir[:, 0])
    assert np.allclose(dr[:, 0], bd[:, 0], rtol=1e-4, atol=1e-5)
