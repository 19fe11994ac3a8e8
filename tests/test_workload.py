"""The seeded workload generator: determinism, slicing, distribution shape."""
import numpy as np

from workload import gen


def test_mix64_known_values():
    # splitmix64 reference outputs for state = 0 + k * GOLDEN (published test vector of the generator, seed 0)
    out = gen.hash_ctr(np.uint64(0), np.arange(1, 4, dtype=np.uint64))
    assert [hex(int(v)) for v in out] == ["0xe220a8397b1dcdaf", "0x6e789e6aa1b965f4", "0x6c45d188009454f"]


def test_rows_are_pure_functions_of_index():
    cfg = gen.CONFIGS["cfg0"]
    a = gen.database(cfg, 0, 300)
    b = gen.database(cfg, 100, 50)
    assert np.array_equal(a[100:150], b)
    c = gen.rows(cfg, 0, 300, chunk=7)
    assert np.array_equal(a, c)
    assert not np.array_equal(gen.queries(cfg, 4), a[:4])
    assert np.array_equal(gen.queries(cfg, 8)[4:], gen.queries(cfg, 4, start=4))


def test_mixture_shape():
    cfg = gen.CONFIGS["cfg0"]
    x = gen.database(cfg, 0, 8192)
    comp = gen.components_of(cfg, np.arange(8192, dtype=np.uint64))
    cen = gen.centres(cfg)
    resid = x - cen[comp]
    assert abs(resid.std() - cfg.sigma) < 0.01
    assert abs(cen.std() - 1.0) < 0.03
    assert np.abs(resid).max() <= 4.9 * cfg.sigma + 1e-6
    counts = np.bincount(comp, minlength=cfg.n_components)
    assert counts.min() > 60 and counts.max() < 200          # uniform weights


def test_zipf_weights():
    cfg = gen.CONFIGS["cfg1"]
    comp = gen.components_of(cfg, np.arange(200_000, dtype=np.uint64))
    counts = np.bincount(comp, minlength=cfg.n_components) / 200_000
    w = np.arange(1, 1025) ** -1.1
    w /= w.sum()
    assert abs(counts[0] - w[0]) < 0.005 and abs(counts[1] - w[1]) < 0.004
    cum = gen.component_cum(cfg)
    assert cum[-1] == 1 << 32 and np.all(np.diff(cum.astype(np.int64)) > 0)


def test_draw_distinct_rows():
    r = gen.draw_distinct_rows(1000, 1000, 3)
    assert sorted(r.tolist()) == list(range(1000))
    r2 = gen.draw_distinct_rows(10**9, 500, 3)
    assert len(set(r2.tolist())) == 500 and r2.max() < 10**9
    assert np.array_equal(r2, gen.draw_distinct_rows(10**9, 500, 3))
    assert not np.array_equal(r2, gen.draw_distinct_rows(10**9, 500, 4))
