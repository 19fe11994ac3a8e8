"""Seeded synthetic workload for IVF-PQ retrieval experiments.

This module only *draws inputs*: database vectors, query vectors and the row
indices a k-means run starts from.  It contains none of the retrieval
method's arithmetic (no distances, no quantisation, no search); the CPU
oracle and the HIP library both consume what it produces.

The database stands in for the paper's 3-billion-chunk sentence-embedding
database (Appendix "Detailed Evaluation Setup", Datasets): a Gaussian mixture
whose components play the role of topics.  Every value is a pure function of
(seed, row, coordinate), so any slice can be regenerated anywhere, and the
recipe uses only integer hashing plus three correctly rounded fp32 operations,
so the numpy implementation here and the on-device generator
(`workload/gen_hip.hip`) agree bit for bit.

Recipe for coordinate t of row i of a configuration with seed s:
  key(stream)   = mix64(s * GOLDEN + stream)
  hash(key, c)  = mix64(key + c * GOLDEN)            (splitmix64 sequence)
  component(i)  = #{ j : cum[j] <= hash(key(COMPONENT), i) >> 32 }
                  with cum = floor(cumsum(weights) * 2^32)
  z(key, c)     = fp32(S - 262140) * INV_STD, S = sum of the eight 16-bit
                  fields of hash(key, 2c) and hash(key, 2c+1)
                  (Irwin-Hall approximation of N(0,1); support +-4.9 sigma)
  centre[j][t]  = z(key(CENTRES), j*d + t)
  x[i][t]       = centre[component(i)][t] (+) sigma (*) z(key(NOISE), i*d + t)
where (+), (*) are single fp32 operations (never fused).
Query q uses row index QUERY_ROW0 + q, which no database row reaches.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

STREAM_CENTRES = 1
STREAM_COMPONENT = 2
STREAM_NOISE = 3
STREAM_KMEANS_INIT = 4

QUERY_ROW0 = 1 << 40
IH_MEAN = 262140                      # 8 * 65535 / 2
INV_STD = np.float32(1.8688123650118534e-05)   # 1 / sqrt(8 * (65536^2 - 1) / 12)


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    seed: int
    n_components: int
    zipf_s: float        # 0.0 -> uniform component weights
    sigma: float
    N: int
    d: int
    nlist: int
    M: int
    train_sample: int
    nq: int
    nprobe: int
    k: int
    kmeans_iters: int = 10

    @property
    def dsub(self) -> int:
        return self.d // self.M

    def scaled(self, **kw) -> "WorkloadConfig":
        return replace(self, **kw)


# The five benchmark configurations (database size, mixture, index shape and
# the search call each is quoted on).
CONFIGS = {
    "cfg0": WorkloadConfig("cfg0", 0, 64, 0.0, 0.3, 65_536, 128, 256, 16, 65_536, 32, 8, 10),
    "cfg1": WorkloadConfig("cfg1", 1, 1024, 1.1, 0.25, 4_194_304, 768, 4096, 64, 262_144, 64, 32, 100),
    "cfg2": WorkloadConfig("cfg2", 2, 1024, 1.1, 0.25, 16_777_216, 768, 16_384, 64, 262_144, 8, 256, 100),
    "cfg3": WorkloadConfig("cfg3", 3, 4096, 1.1, 0.25, 268_435_456, 768, 65_536, 64, 1_048_576, 64, 64, 100),
    "cfg4": WorkloadConfig("cfg4", 4, 4096, 1.1, 0.25, 1_073_741_824, 768, 65_536, 64, 1_048_576, 256, 128, 100),
    # the shape of the paper's own database (Appendix "Detailed Evaluation Setup": three billion 384-dimensional
    # vectors, 16,384 lists, 64-byte codes, nprobe 64, the k = 2 neighbours RETRO retrieves per chunk)
    "paper": WorkloadConfig("paper", 5, 4096, 1.1, 0.25, 3_000_000_000, 384, 16_384, 64, 1_048_576, 64, 64, 2),
}


def mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on uint64 arrays (wrap-around arithmetic)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def stream_key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        return mix64(np.uint64(seed) * GOLDEN + np.uint64(stream))[()]


def hash_ctr(key: np.uint64, ctr: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        return mix64(np.uint64(key) + np.asarray(ctr, dtype=np.uint64) * GOLDEN)


def _fields16(h: np.ndarray) -> np.ndarray:
    m = np.uint64(0xFFFF)
    return ((h & m) + ((h >> np.uint64(16)) & m) + ((h >> np.uint64(32)) & m)
            + (h >> np.uint64(48))).astype(np.int64)


def variate(key: np.uint64, ctr: np.ndarray) -> np.ndarray:
    """Approximately N(0,1) fp32 variate for each counter (integer sum, one multiply)."""
    ctr = np.asarray(ctr, dtype=np.uint64)
    two = np.uint64(2)
    s = _fields16(hash_ctr(key, ctr * two)) + _fields16(hash_ctr(key, ctr * two + np.uint64(1)))
    return (s - IH_MEAN).astype(np.float32) * INV_STD


def component_cum(cfg: WorkloadConfig) -> np.ndarray:
    """Cumulative component weights scaled to 2^32 (uint64, last entry == 2^32)."""
    r = np.arange(1, cfg.n_components + 1, dtype=np.float64)
    w = np.ones_like(r) if cfg.zipf_s == 0.0 else r ** (-cfg.zipf_s)
    cum = np.floor(np.cumsum(w) / np.sum(w) * 4294967296.0).astype(np.uint64)
    cum[-1] = np.uint64(1 << 32)
    return cum


def centres(cfg: WorkloadConfig) -> np.ndarray:
    """Mixture centres, fp32 [n_components, d]."""
    key = stream_key(cfg.seed, STREAM_CENTRES)
    ctr = np.arange(cfg.n_components * cfg.d, dtype=np.uint64)
    return variate(key, ctr).reshape(cfg.n_components, cfg.d)


def components_of(cfg: WorkloadConfig, rows: np.ndarray, cum: np.ndarray | None = None) -> np.ndarray:
    cum = component_cum(cfg) if cum is None else cum
    u = hash_ctr(stream_key(cfg.seed, STREAM_COMPONENT), rows) >> np.uint64(32)
    return np.searchsorted(cum, u, side="right").astype(np.int32)


def rows(cfg: WorkloadConfig, row0: int, count: int, chunk: int = 8192) -> np.ndarray:
    """fp32 [count, d]: rows row0 .. row0+count-1 of the configuration's row space."""
    cum = component_cum(cfg)
    cen = centres(cfg)
    key = stream_key(cfg.seed, STREAM_NOISE)
    sigma = np.float32(cfg.sigma)
    out = np.empty((count, cfg.d), dtype=np.float32)
    t = np.arange(cfg.d, dtype=np.uint64)[None, :]
    for a in range(0, count, chunk):
        b = min(count, a + chunk)
        r = np.arange(row0 + a, row0 + b, dtype=np.uint64)
        comp = components_of(cfg, r, cum)
        z = variate(key, r[:, None] * np.uint64(cfg.d) + t)
        noise = sigma * z                      # one fp32 multiply
        out[a:b] = cen[comp] + noise           # one fp32 add
    return out


def database(cfg: WorkloadConfig, start: int = 0, count: int | None = None) -> np.ndarray:
    count = cfg.N - start if count is None else count
    assert 0 <= start and start + count <= cfg.N
    return rows(cfg, start, count)


def queries(cfg: WorkloadConfig, nq: int | None = None, start: int = 0) -> np.ndarray:
    nq = cfg.nq if nq is None else nq
    return rows(cfg, QUERY_ROW0 + start, nq)


def draw_distinct_rows(S: int, K: int, seed: int) -> np.ndarray:
    """K distinct integers from [0, S): the first K steps of a Fisher-Yates
    shuffle of 0..S-1 driven by hash(key(seed, KMEANS_INIT), step).  int64 [K]."""
    assert 0 < K <= S
    key = stream_key(seed, STREAM_KMEANS_INIT)
    h = hash_ctr(key, np.arange(K, dtype=np.uint64))
    swapped: dict[int, int] = {}
    out = np.empty(K, dtype=np.int64)
    for i in range(K):
        j = i + int(h[i] % np.uint64(S - i))
        vi = swapped.get(i, i)
        vj = swapped.get(j, j)
        out[i] = vj
        swapped[j] = vi
    return out
