"""CPU oracle for IVF-PQ retrieval: ctypes front end of `ivfpq_oracle.c`.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only
the tests, the smoke check and the benchmark's CPU-baseline leg do.  The
oracle shares no code with the HIP library (the index-file layout written by
`write_index_file` is an interface, restated independently on each side).

Every function cites the part of the method it follows in the C source.
Pins (see tests/test_oracle_*.py): brute-force exact kNN on tiny inputs,
identity codebooks with nprobe = nlist reducing to exact search, ADC equal to
the distance to the decoded vector, recall / candidate-set monotonicity in
nprobe, a worked two-sub-quantiser table, and k-means closed forms.
"""
from __future__ import annotations

import ctypes as C
import os
import struct
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ivfpq_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, strict IEEE arithmetic, OpenMP threads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = f"{_LIB}.{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-ftree-vectorize", "-march=x86-64-v3", "-fno-fast-math",
                               "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


# --------------------------------------------------------------------------
def assign(x: np.ndarray, c: np.ndarray, return_dist: bool = False):
    """argmin_j ||x_i - c_j||^2 (fp32-rounded values, lowest j on ties)."""
    x = _f32(x); c = _f32(c)
    n, d = x.shape
    idx = np.empty(n, dtype=np.int32)
    dist = np.empty(n, dtype=np.float32) if return_dist else None
    _load().oracle_assign(_p(x, C.c_float), C.c_int64(n), C.c_int(d), C.c_int64(d), _p(c, C.c_float),
                          C.c_int64(c.shape[0]), _p(idx, C.c_int32), _p(dist, C.c_float))
    return (idx, dist) if return_dist else idx


def assign_among(x: np.ndarray, c: np.ndarray, cand: np.ndarray, return_dist: bool = False):
    """Nearest centre of each row among the centres listed for it (cand: int32 [n, T], negative entries skipped)."""
    x = _f32(x); c = _f32(c)
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    n, d = x.shape
    assert cand.ndim == 2 and cand.shape[0] == n and cand.max(initial=-1) < c.shape[0] and np.all((cand >= 0).any(axis=1))
    idx = np.empty(n, dtype=np.int32)
    dist = np.empty(n, dtype=np.float32) if return_dist else None
    _load().oracle_assign_among(_p(x, C.c_float), C.c_int64(n), C.c_int(d), C.c_int64(d), _p(c, C.c_float),
                                _p(cand, C.c_int32), C.c_int(cand.shape[1]), _p(idx, C.c_int32), _p(dist, C.c_float))
    return (idx, dist) if return_dist else idx


def encode_codes(x: np.ndarray, pq: np.ndarray) -> np.ndarray:
    """PQ codes uint8 [n, M] of each row of x (the code part of `encode`, without the list assignment)."""
    x = _f32(x); pq = _f32(pq)
    n, d = x.shape
    M, ksub, dsub = pq.shape
    assert M * dsub == d and ksub <= 256
    codes = np.empty((n, M), dtype=np.uint8)
    _load().oracle_encode(_p(x, C.c_float), C.c_int64(n), C.c_int(d), None, C.c_int64(0), _p(pq, C.c_float), C.c_int(M),
                          C.c_int(ksub), None, _p(codes, C.c_uint8))
    return codes


def kmeans(x: np.ndarray, K: int, init_rows: np.ndarray, iters: int = 10, return_inertia: bool = False):
    """Fixed-iteration Lloyd k-means started from rows `init_rows` of x.  x may be a strided view
    (rows contiguous in their last dimension)."""
    assert x.dtype == np.float32 and x.ndim == 2 and x.strides[1] == 4
    S, d = x.shape
    ldx = x.strides[0] // 4
    init_rows = np.ascontiguousarray(init_rows, dtype=np.int64)
    assert init_rows.shape == (K,) and len(np.unique(init_rows)) == K
    c = np.empty((K, d), dtype=np.float32)
    inertia = np.empty(iters, dtype=np.float64)
    _load().oracle_kmeans(C.c_void_p(x.ctypes.data), C.c_int64(S), C.c_int(d), C.c_int64(ldx), C.c_int64(K),
                          C.c_int(iters), _p(init_rows, C.c_int64), _p(c, C.c_float), _p(inertia, C.c_double))
    return (c, inertia) if return_inertia else c


def encode(x: np.ndarray, coarse: np.ndarray, pq: np.ndarray):
    """(list number int32 [n], PQ codes uint8 [n, M]) of each row of x.  pq: [M, ksub, dsub]."""
    x = _f32(x); coarse = _f32(coarse); pq = _f32(pq)
    n, d = x.shape
    M, ksub, dsub = pq.shape
    assert M * dsub == d and ksub <= 256
    lists = np.empty(n, dtype=np.int32)
    codes = np.empty((n, M), dtype=np.uint8)
    _load().oracle_encode(_p(x, C.c_float), C.c_int64(n), C.c_int(d), _p(coarse, C.c_float),
                          C.c_int64(coarse.shape[0]), _p(pq, C.c_float), C.c_int(M), C.c_int(ksub),
                          _p(lists, C.c_int32), _p(codes, C.c_uint8))
    return lists, codes


@dataclass
class Index:
    """An IVF-PQ index in canonical form: list l = entries list_off[l]:list_off[l+1] of `codes`/`ids`,
    in ascending id order."""
    coarse: np.ndarray      # [nlist, d] f32
    pq: np.ndarray          # [M, ksub, dsub] f32
    list_off: np.ndarray    # [nlist + 1] i64
    codes: np.ndarray       # [ntotal, M] u8
    ids: np.ndarray         # [ntotal] i64
    residual: bool = False  # codes quantise x - centre of x's list instead of x

    @property
    def nlist(self): return self.coarse.shape[0]
    @property
    def d(self): return self.coarse.shape[1]
    @property
    def M(self): return self.pq.shape[0]
    @property
    def ntotal(self): return self.codes.shape[0]


def build_lists(lists: np.ndarray, codes: np.ndarray, ids: np.ndarray, nlist: int):
    """Group encoded vectors by list; inside a list, ascending id."""
    order = np.lexsort((ids, lists))
    counts = np.bincount(lists, minlength=nlist).astype(np.int64)
    off = np.zeros(nlist + 1, dtype=np.int64)
    np.cumsum(counts, out=off[1:])
    return off, np.ascontiguousarray(codes[order]), np.ascontiguousarray(ids[order].astype(np.int64))


def train(sample: np.ndarray, nlist: int, M: int, coarse_init: np.ndarray, pq_init: list, iters: int = 10,
          ksub: int = 256):
    """Coarse centres = k-means(sample, nlist); codebook m = k-means(m-th slice of sample, ksub)."""
    sample = _f32(sample)
    d = sample.shape[1]
    dsub = d // M
    coarse = kmeans(sample, nlist, coarse_init, iters)
    pq = np.empty((M, ksub, dsub), dtype=np.float32)
    for m in range(M):
        pq[m] = kmeans(sample[:, m * dsub:(m + 1) * dsub], ksub, pq_init[m], iters)
    return coarse, pq


def make_index(x: np.ndarray, coarse: np.ndarray, pq: np.ndarray, ids: np.ndarray | None = None) -> Index:
    lists, codes = encode(x, coarse, pq)
    ids = np.arange(x.shape[0], dtype=np.int64) if ids is None else np.asarray(ids, dtype=np.int64)
    off, codes, ids = build_lists(lists, codes, ids, coarse.shape[0])
    return Index(_f32(coarse), _f32(pq), off, codes, ids)


# --------------------------------------------------------------------------
def coarse_search(q: np.ndarray, coarse: np.ndarray, nprobe: int):
    q = _f32(q); coarse = _f32(coarse)
    nq, d = q.shape
    probes = np.empty((nq, nprobe), dtype=np.int32)
    dist = np.empty((nq, nprobe), dtype=np.float32)
    _load().oracle_coarse(_p(q, C.c_float), C.c_int64(nq), C.c_int(d), _p(coarse, C.c_float),
                          C.c_int64(coarse.shape[0]), C.c_int(nprobe), _p(probes, C.c_int32), _p(dist, C.c_float))
    return probes, dist


def lut(q: np.ndarray, pq: np.ndarray) -> np.ndarray:
    q = _f32(q); pq = _f32(pq)
    nq, d = q.shape
    M, ksub, dsub = pq.shape
    out = np.empty((nq, M, ksub), dtype=np.float32)
    _load().oracle_lut(_p(q, C.c_float), C.c_int64(nq), C.c_int(d), _p(pq, C.c_float), C.c_int(M), C.c_int(ksub),
                       _p(out, C.c_float))
    return out


def search_with_probes(index: Index, q: np.ndarray, probes: np.ndarray, k: int):
    q = _f32(q)
    nq, d = q.shape
    probes = np.ascontiguousarray(probes, dtype=np.int32)
    nprobe = probes.shape[1]
    M, ksub, dsub = index.pq.shape
    od = np.empty((nq, k), dtype=np.float32)
    oi = np.empty((nq, k), dtype=np.int64)
    scanned = np.empty(nq, dtype=np.int64)
    _load().oracle_search_with_probes(
        _p(q, C.c_float), C.c_int64(nq), C.c_int(d), _p(index.pq, C.c_float), C.c_int(M), C.c_int(ksub),
        _p(index.list_off, C.c_int64), _p(index.codes, C.c_uint8), _p(index.ids, C.c_int64),
        _p(probes, C.c_int32), C.c_int(nprobe), C.c_int(k), _p(od, C.c_float), _p(oi, C.c_int64),
        _p(scanned, C.c_int64))
    return od, oi, scanned


def scan_with_probes(index: Index, q_row: np.ndarray, probes_row: np.ndarray):
    """Distance and id of every vector in one query's probed lists, in probe order, with no selection:
    (dist [ncand] f32, ids [ncand] i64).  The arithmetic is that of search_with_probes."""
    q_row = _f32(q_row).reshape(-1)
    probes_row = np.ascontiguousarray(probes_row, dtype=np.int32).reshape(-1)
    M, ksub, dsub = index.pq.shape
    lens = np.diff(index.list_off)
    ncand = int(lens[probes_row[probes_row >= 0]].sum())
    od = np.empty(ncand, dtype=np.float32)
    oi = np.empty(ncand, dtype=np.int64)
    fn = _load().oracle_scan_with_probes
    fn.restype = C.c_int64
    got = fn(_p(q_row, C.c_float), C.c_int(q_row.shape[0]), _p(index.pq, C.c_float), C.c_int(M), C.c_int(ksub),
             _p(index.list_off, C.c_int64), _p(index.codes, C.c_uint8), _p(index.ids, C.c_int64),
             _p(probes_row, C.c_int32), C.c_int(probes_row.shape[0]), _p(od, C.c_float), _p(oi, C.c_int64))
    assert got == ncand
    return od, oi


# --------------------------------------------------------------------------
# Residual variant: codes quantise x - centre of x's list; `Index.residual` marks such an index.
def residuals(x: np.ndarray, coarse: np.ndarray, lists: np.ndarray) -> np.ndarray:
    x = _f32(x); coarse = _f32(coarse)
    lists = np.ascontiguousarray(lists, dtype=np.int32)
    out = np.empty_like(x)
    _load().oracle_residuals(_p(x, C.c_float), C.c_int64(x.shape[0]), C.c_int(x.shape[1]), _p(coarse, C.c_float),
                             _p(lists, C.c_int32), _p(out, C.c_float))
    return out


def encode_residual(x: np.ndarray, coarse: np.ndarray, pq: np.ndarray):
    x = _f32(x); coarse = _f32(coarse); pq = _f32(pq)
    n, d = x.shape
    M, ksub, dsub = pq.shape
    lists = np.empty(n, dtype=np.int32)
    codes = np.empty((n, M), dtype=np.uint8)
    _load().oracle_encode_residual(_p(x, C.c_float), C.c_int64(n), C.c_int(d), _p(coarse, C.c_float),
                                   C.c_int64(coarse.shape[0]), _p(pq, C.c_float), C.c_int(M), C.c_int(ksub),
                                   _p(lists, C.c_int32), _p(codes, C.c_uint8))
    return lists, codes


def train_residual(sample: np.ndarray, nlist: int, M: int, coarse_init: np.ndarray, pq_init: list, iters: int = 10,
                   ksub: int = 256):
    """Coarse centres = k-means(sample, nlist); codebook m = k-means(m-th slice of the sample's residuals, ksub)."""
    sample = _f32(sample)
    d = sample.shape[1]
    dsub = d // M
    coarse = kmeans(sample, nlist, coarse_init, iters)
    r = residuals(sample, coarse, assign(sample, coarse))
    pq = np.empty((M, ksub, dsub), dtype=np.float32)
    for m in range(M):
        pq[m] = kmeans(r[:, m * dsub:(m + 1) * dsub], ksub, pq_init[m], iters)
    return coarse, pq


def make_index_residual(x: np.ndarray, coarse: np.ndarray, pq: np.ndarray, ids: np.ndarray | None = None) -> Index:
    lists, codes = encode_residual(x, coarse, pq)
    ids = np.arange(x.shape[0], dtype=np.int64) if ids is None else np.asarray(ids, dtype=np.int64)
    off, codes, ids = build_lists(lists, codes, ids, coarse.shape[0])
    return Index(_f32(coarse), _f32(pq), off, codes, ids, residual=True)


def search_residual_with_probes(index: Index, q: np.ndarray, probes: np.ndarray, k: int):
    q = _f32(q)
    nq, d = q.shape
    probes = np.ascontiguousarray(probes, dtype=np.int32)
    M, ksub, dsub = index.pq.shape
    od = np.empty((nq, k), dtype=np.float32)
    oi = np.empty((nq, k), dtype=np.int64)
    _load().oracle_search_residual_with_probes(
        _p(q, C.c_float), C.c_int64(nq), C.c_int(d), _p(index.coarse, C.c_float), _p(index.pq, C.c_float), C.c_int(M),
        C.c_int(ksub), _p(index.list_off, C.c_int64), _p(index.codes, C.c_uint8), _p(index.ids, C.c_int64),
        _p(probes, C.c_int32), C.c_int(probes.shape[1]), C.c_int(k), _p(od, C.c_float), _p(oi, C.c_int64))
    lens = np.diff(index.list_off)
    scanned = np.array([int(lens[p[p >= 0]].sum()) for p in probes], dtype=np.int64)
    return od, oi, scanned


def scan_residual_with_probes(index: Index, q_row: np.ndarray, probes_row: np.ndarray):
    q_row = _f32(q_row).reshape(-1)
    probes_row = np.ascontiguousarray(probes_row, dtype=np.int32).reshape(-1)
    M, ksub, dsub = index.pq.shape
    lens = np.diff(index.list_off)
    ncand = int(lens[probes_row[probes_row >= 0]].sum())
    od = np.empty(ncand, dtype=np.float32)
    oi = np.empty(ncand, dtype=np.int64)
    fn = _load().oracle_scan_residual_with_probes
    fn.restype = C.c_int64
    got = fn(_p(q_row, C.c_float), C.c_int(q_row.shape[0]), _p(index.coarse, C.c_float), _p(index.pq, C.c_float), C.c_int(M),
             C.c_int(ksub), _p(index.list_off, C.c_int64), _p(index.codes, C.c_uint8), _p(index.ids, C.c_int64),
             _p(probes_row, C.c_int32), C.c_int(probes_row.shape[0]), _p(od, C.c_float), _p(oi, C.c_int64))
    assert got == ncand
    return od, oi


def search(index: Index, q: np.ndarray, nprobe: int, k: int):
    """(dist [nq,k] f32, ids [nq,k] i64, probes [nq,nprobe] i32, scanned [nq] i64)."""
    q = _f32(q)
    if index.residual:
        probes, _ = coarse_search(q, index.coarse, nprobe)
        od, oi, scanned = search_residual_with_probes(index, q, probes, k)
        return od, oi, probes, scanned
    nq, d = q.shape
    M, ksub, dsub = index.pq.shape
    od = np.empty((nq, k), dtype=np.float32)
    oi = np.empty((nq, k), dtype=np.int64)
    probes = np.empty((nq, nprobe), dtype=np.int32)
    scanned = np.empty(nq, dtype=np.int64)
    _load().oracle_search(
        _p(q, C.c_float), C.c_int64(nq), C.c_int(d), _p(index.coarse, C.c_float), C.c_int64(index.nlist),
        _p(index.pq, C.c_float), C.c_int(M), C.c_int(ksub), _p(index.list_off, C.c_int64),
        _p(index.codes, C.c_uint8), _p(index.ids, C.c_int64), C.c_int(nprobe), C.c_int(k),
        _p(od, C.c_float), _p(oi, C.c_int64), _p(probes, C.c_int32), _p(scanned, C.c_int64))
    return od, oi, probes, scanned


def brute_force_knn(x: np.ndarray, q: np.ndarray, k: int):
    x = _f32(x); q = _f32(q)
    nq = q.shape[0]
    od = np.empty((nq, k), dtype=np.float32)
    oi = np.empty((nq, k), dtype=np.int64)
    _load().oracle_brute_force_knn(_p(x, C.c_float), C.c_int64(x.shape[0]), C.c_int(x.shape[1]), _p(q, C.c_float),
                                   C.c_int64(nq), C.c_int(k), _p(od, C.c_float), _p(oi, C.c_int64))
    return od, oi


def decode(codes: np.ndarray, pq: np.ndarray) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    pq = _f32(pq)
    M, ksub, dsub = pq.shape
    n = codes.shape[0]
    out = np.empty((n, M * dsub), dtype=np.float32)
    _load().oracle_decode(_p(codes, C.c_uint8), C.c_int64(n), _p(pq, C.c_float), C.c_int(M), C.c_int(ksub),
                          C.c_int(dsub), _p(out, C.c_float))
    return out


def recall_at_k(ann_ids: np.ndarray, exact_ids: np.ndarray) -> float:
    """Mean over queries of |ANN_k intersect exact_k| / k (reading: the paper names recall without defining it)."""
    hits = [len(set(a[a >= 0].tolist()) & set(e.tolist())) for a, e in zip(ann_ids, exact_ids)]
    return float(np.mean(hits)) / exact_ids.shape[1]


# --------------------------------------------------------------------------
def write_index_file(index: Index, path: str) -> None:
    """Little-endian index file: 64-byte header ("PRAGIVF1", u32 version=1, d, nlist, M, nbits=8, 0,
    u64 ntotal, zero padding), centres f32 [nlist*d], codebooks f32 [M*256*dsub], list lengths i64 [nlist],
    codes u8 [ntotal*M] list-major, ids i64 [ntotal]."""
    M, ksub, dsub = index.pq.shape
    assert ksub == 256
    hdr = b"PRAGIVF1" + struct.pack("<6IQ", 1, index.d, index.nlist, M, 8, 0, index.ntotal)
    hdr += b"\0" * (64 - len(hdr))
    with open(path, "wb") as f:
        f.write(hdr)
        f.write(index.coarse.astype("<f4").tobytes())
        f.write(index.pq.astype("<f4").tobytes())
        f.write(np.diff(index.list_off).astype("<i8").tobytes())
        f.write(index.codes.tobytes())
        f.write(index.ids.astype("<i8").tobytes())
