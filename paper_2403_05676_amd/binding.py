"""ctypes binding of the C ABI declared in include/piperag.h (same names, argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpiperag.so")
_lib = None

NSTAGES = 4
STAGE_NAMES = ("coarse", "select+plan", "lut", "scan+merge")


class PiperagError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"piperag error {code}: {msg}")
        self.code = code


class Params(C.Structure):
    _fields_ = [("d", C.c_int32), ("nlist", C.c_int32), ("M", C.c_int32), ("nbits", C.c_int32),
                ("ntotal", C.c_int64), ("max_nq", C.c_int32), ("max_nprobe", C.c_int32), ("max_k", C.c_int32),
                ("residual", C.c_int32)]


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> C.CDLL:
    """Loads libpiperag.so built in-tree (python -m paper_2403_05676_amd.build or __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2403_05676_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    sig = {
        "piperag_ivf_load": [C.c_char_p, C.POINTER(Params), C.POINTER(vp)],
        "piperag_ivf_create": [C.POINTER(Params), vp, vp, C.POINTER(vp)],
        "piperag_kmeans": [vp, i64, i32, i64, i32, i32, vp, vp, vp, vp],
        "piperag_ivf_add": [vp, vp, i64, vp, vp],
        "piperag_ivf_add_encoded": [vp, vp, vp, vp, i64, vp],
        "piperag_ivf_finalize": [vp, vp],
        "piperag_ivf_count": [vp, vp, i64, vp],
        "piperag_ivf_reserve": [vp, vp],
        "piperag_ivf_place": [vp, vp, i64, vp, vp],
        "piperag_ivf_save": [vp, C.c_char_p],
        "piperag_ivfpq_search": [vp, vp, i32, i32, i32, vp, vp, vp],
        "piperag_ivfpq_search_static": [vp, vp, i32, i32, i32, vp, vp, vp],
        "piperag_latency_profile": [vp, vp, i32, vp, i32, i32, i32, vp, vp, vp],
        "piperag_max_nprobe": [vp, C.c_float, C.c_float, i32, vp, vp, vp],
        "piperag_project_latency": [vp, vp, i32, C.c_float, C.c_float, vp, vp],
        "piperag_ivf_coarse": [vp, vp, i32, i32, vp, vp, vp],
        "piperag_ivf_lut": [vp, vp, i32, vp, vp],
        "piperag_ivfpq_search_probes": [vp, vp, i32, vp, i32, i32, vp, vp, vp],
        "piperag_ivf_encode": [vp, vp, i64, vp, vp, vp],
        "piperag_ivf_get_list": [vp, i32, C.POINTER(i64), vp, vp],
        "piperag_ivf_list_lengths": [vp, vp],
        "piperag_search_stats": [vp, C.POINTER(i64), C.POINTER(i64)],
        "piperag_set_stage_timing": [vp, C.c_int],
        "piperag_set_graph_replay": [vp, C.c_int],
        "piperag_set_scan_streaming": [vp, C.c_int],
        "piperag_set_compute_units": [vp, i32],
        "piperag_stage_times": [vp, vp],
        "piperag_stream_create_cu_slice": [i32, i32, C.POINTER(vp)],
        "piperag_stream_destroy": [vp],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.piperag_ivf_free.argtypes = [vp]
    lib.piperag_ivf_free.restype = None
    lib.piperag_ivf_ntotal.argtypes = [vp]
    lib.piperag_ivf_ntotal.restype = i64
    lib.piperag_last_error.argtypes = []
    lib.piperag_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise PiperagError(rc, load_library().piperag_last_error().decode(errors="replace"))


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype: torch.dtype) -> int:
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"expected a contiguous CUDA tensor of {dtype}, got {t.dtype} on {t.device}")
    return t.data_ptr()


def max_nprobe(fit, budget_ms: float, nprobe_cap: int, overhead_ms: float = 0.0):
    """piperag_max_nprobe: (nprobe, fits, predicted_ms)."""
    f = np.ascontiguousarray(fit, dtype=np.float32)
    assert f.shape == (2,)
    npr, fits, pred = C.c_int32(), C.c_int32(), C.c_float()
    _check(load_library().piperag_max_nprobe(f.ctypes.data, float(overhead_ms), float(budget_ms), int(nprobe_cap),
                                             C.addressof(npr), C.addressof(fits), C.addressof(pred)))
    return npr.value, bool(fits.value), pred.value


def project_latency(inference_ms, retrieval_ms, inference_speedup: float = 1.0, retrieval_speedup: float = 1.0):
    """piperag_project_latency: (sequential_ms, pipelined_ms)."""
    ti = np.ascontiguousarray(inference_ms, dtype=np.float32)
    tr = np.ascontiguousarray(retrieval_ms, dtype=np.float32)
    assert ti.ndim == 1 and ti.shape == tr.shape
    seq, pipe = C.c_double(), C.c_double()
    _check(load_library().piperag_project_latency(ti.ctypes.data, tr.ctypes.data, ti.shape[0], float(inference_speedup),
                                                  float(retrieval_speedup), C.addressof(seq), C.addressof(pipe)))
    return seq.value, pipe.value


def stream_create_cu_slice(first_cu: int, ncu: int) -> torch.cuda.ExternalStream:
    """piperag_stream_create_cu_slice, wrapped for torch (the handle stays valid until stream_destroy)."""
    h = C.c_void_p()
    _check(load_library().piperag_stream_create_cu_slice(int(first_cu), int(ncu), C.byref(h)))
    return torch.cuda.ExternalStream(h.value)


def stream_destroy(stream: torch.cuda.ExternalStream) -> None:
    _check(load_library().piperag_stream_destroy(C.c_void_p(stream.cuda_stream)))


def kmeans(x: torch.Tensor, K: int, init_rows: np.ndarray, iters: int = 10, return_inertia: bool = False):
    """piperag_kmeans on a 2-D float32 CUDA tensor (rows may be strided: a column slice of a wider matrix)."""
    if not (x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.stride(1) == 1):
        raise TypeError("expected a 2-D float32 CUDA tensor with unit column stride")
    n, d = x.shape
    rows = np.ascontiguousarray(init_rows, dtype=np.int64)
    if rows.shape != (K,):
        raise ValueError("init_rows must hold K row numbers")
    out = torch.empty((K, d), dtype=torch.float32, device=x.device)
    inertia = np.empty(iters, dtype=np.float64) if return_inertia else None
    _check(load_library().piperag_kmeans(x.data_ptr(), n, d, x.stride(0), K, iters, rows.ctypes.data, out.data_ptr(),
                                         inertia.ctypes.data if return_inertia else None, _stream()))
    return (out, inertia) if return_inertia else out


class Index:
    """Owns one `piperag_index`.  Method names follow the C entry points (piperag_<name>)."""

    def __init__(self, handle: int, d: int, nlist: int, M: int):
        self._h = C.c_void_p(handle)
        self.d, self.nlist, self.M = d, nlist, M

    # ---- life cycle --------------------------------------------------------------------------
    @staticmethod
    def ivf_create(centroids: np.ndarray, pq_codebook: np.ndarray, capacity: int, max_nq: int = 256,
                   max_nprobe: int = 256, max_k: int = 128, residual: bool = False) -> "Index":
        cent = np.ascontiguousarray(centroids, dtype=np.float32)
        pq = np.ascontiguousarray(pq_codebook, dtype=np.float32)
        nlist, d = cent.shape
        M, ksub, dsub = pq.shape
        if ksub != 256 or M * dsub != d:
            raise ValueError("codebook must be [M, 256, d/M]")
        p = Params(d, nlist, M, 8, capacity, max_nq, min(max_nprobe, nlist), max_k, int(residual))
        h = C.c_void_p()
        _check(load_library().piperag_ivf_create(C.byref(p), cent.ctypes.data, pq.ctypes.data, C.byref(h)))
        return Index(h.value, d, nlist, M)

    @staticmethod
    def ivf_load(path: str, max_nq: int = 256, max_nprobe: int = 256, max_k: int = 128) -> "Index":
        p = Params(0, 0, 0, 8, 0, max_nq, max_nprobe, max_k, 0)
        h = C.c_void_p()
        _check(load_library().piperag_ivf_load(path.encode(), C.byref(p), C.byref(h)))
        # read the shape back from the file header
        with open(path, "rb") as f:
            hdr = np.frombuffer(f.read(32), dtype="<u4")
        return Index(h.value, int(hdr[3]), int(hdr[4]), int(hdr[5]))

    def ivf_free(self) -> None:
        if self._h:
            load_library().piperag_ivf_free(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.ivf_free()
        except Exception:
            pass

    def ivf_add(self, x: torch.Tensor, ids: torch.Tensor | None = None) -> None:
        n = x.shape[0]
        _check(load_library().piperag_ivf_add(self._h, _dev(x, torch.float32), n,
                                              _dev(ids, torch.int64) if ids is not None else None, _stream()))

    def ivf_add_encoded(self, lists: torch.Tensor, codes: torch.Tensor, ids: torch.Tensor | None = None) -> None:
        n = lists.shape[0]
        _check(load_library().piperag_ivf_add_encoded(self._h, _dev(lists, torch.int32), _dev(codes, torch.uint8),
                                                      _dev(ids, torch.int64) if ids is not None else None, n, _stream()))

    def ivf_count(self, x: torch.Tensor) -> None:
        _check(load_library().piperag_ivf_count(self._h, _dev(x, torch.float32), x.shape[0], _stream()))

    def ivf_reserve(self) -> None:
        _check(load_library().piperag_ivf_reserve(self._h, _stream()))

    def ivf_place(self, x: torch.Tensor, ids: torch.Tensor | None = None) -> None:
        _check(load_library().piperag_ivf_place(self._h, _dev(x, torch.float32), x.shape[0],
                                                _dev(ids, torch.int64) if ids is not None else None, _stream()))

    def ivf_finalize(self) -> None:
        _check(load_library().piperag_ivf_finalize(self._h, _stream()))

    def ivf_save(self, path: str) -> None:
        _check(load_library().piperag_ivf_save(self._h, path.encode()))

    def ivf_ntotal(self) -> int:
        return int(load_library().piperag_ivf_ntotal(self._h))

    # ---- search ------------------------------------------------------------------------------
    def ivfpq_search(self, queries: torch.Tensor, nprobe: int, k: int, out_dist: torch.Tensor | None = None,
                     out_ids: torch.Tensor | None = None):
        nq = queries.shape[0]
        if out_dist is None:
            out_dist = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
        if out_ids is None:
            out_ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
        _check(load_library().piperag_ivfpq_search(self._h, _dev(queries, torch.float32), nq, nprobe, k,
                                                   _dev(out_dist, torch.float32), _dev(out_ids, torch.int64), _stream()))
        return out_dist, out_ids

    def ivfpq_search_static(self, queries: torch.Tensor, nprobe: int, k: int, out_dist: torch.Tensor, out_ids: torch.Tensor):
        """piperag_ivfpq_search_static: the caller passes every buffer; nothing is allocated on either side."""
        _check(load_library().piperag_ivfpq_search_static(self._h, _dev(queries, torch.float32), queries.shape[0], nprobe, k,
                                                          _dev(out_dist, torch.float32), _dev(out_ids, torch.int64), _stream()))
        return out_dist, out_ids

    def ivfpq_search_probes(self, queries: torch.Tensor, probes: torch.Tensor, k: int):
        nq, nprobe = probes.shape
        out_dist = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
        out_ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
        _check(load_library().piperag_ivfpq_search_probes(self._h, _dev(queries, torch.float32), nq,
                                                          _dev(probes, torch.int32), nprobe, k,
                                                          _dev(out_dist, torch.float32), _dev(out_ids, torch.int64), _stream()))
        return out_dist, out_ids

    def latency_profile(self, queries: torch.Tensor, nprobes, k: int, reps: int = 20):
        npr = np.ascontiguousarray(nprobes, dtype=np.int32)
        p50 = np.empty(len(npr), dtype=np.float32)
        fit = np.empty(2, dtype=np.float32)
        _check(load_library().piperag_latency_profile(self._h, _dev(queries, torch.float32), queries.shape[0],
                                                      npr.ctypes.data, len(npr), k, reps, p50.ctypes.data, fit.ctypes.data,
                                                      _stream()))
        return p50, fit

    # ---- stage taps --------------------------------------------------------------------------
    def ivf_coarse(self, queries: torch.Tensor, nprobe: int):
        nq = queries.shape[0]
        lists = torch.empty((nq, nprobe), dtype=torch.int32, device=queries.device)
        dist = torch.empty((nq, nprobe), dtype=torch.float32, device=queries.device)
        _check(load_library().piperag_ivf_coarse(self._h, _dev(queries, torch.float32), nq, nprobe,
                                                 _dev(lists, torch.int32), _dev(dist, torch.float32), _stream()))
        return lists, dist

    def ivf_lut(self, queries: torch.Tensor) -> torch.Tensor:
        nq = queries.shape[0]
        out = torch.empty((nq, self.M, 256), dtype=torch.float32, device=queries.device)
        _check(load_library().piperag_ivf_lut(self._h, _dev(queries, torch.float32), nq, _dev(out, torch.float32), _stream()))
        return out

    def ivf_encode(self, x: torch.Tensor):
        n = x.shape[0]
        lists = torch.empty((n,), dtype=torch.int32, device=x.device)
        codes = torch.empty((n, self.M), dtype=torch.uint8, device=x.device)
        _check(load_library().piperag_ivf_encode(self._h, _dev(x, torch.float32), n, _dev(lists, torch.int32),
                                                 _dev(codes, torch.uint8), _stream()))
        return lists, codes

    def ivf_get_list(self, l: int):
        n = C.c_int64()
        _check(load_library().piperag_ivf_get_list(self._h, l, C.byref(n), None, None))
        codes = np.empty((n.value, self.M), dtype=np.uint8)
        ids = np.empty(n.value, dtype=np.int64)
        if n.value:
            _check(load_library().piperag_ivf_get_list(self._h, l, C.byref(n), codes.ctypes.data, ids.ctypes.data))
        return codes, ids

    def ivf_list_lengths(self) -> np.ndarray:
        out = np.empty(self.nlist, dtype=np.int64)
        _check(load_library().piperag_ivf_list_lengths(self._h, out.ctypes.data))
        return out

    def search_stats(self):
        v, b = C.c_int64(), C.c_int64()
        _check(load_library().piperag_search_stats(self._h, C.byref(v), C.byref(b)))
        return v.value, b.value

    def set_stage_timing(self, enable: bool) -> None:
        _check(load_library().piperag_set_stage_timing(self._h, int(enable)))

    def set_graph_replay(self, enable: bool) -> None:
        _check(load_library().piperag_set_graph_replay(self._h, int(enable)))

    def set_scan_streaming(self, mode: int) -> None:
        _check(load_library().piperag_set_scan_streaming(self._h, int(mode)))

    def set_compute_units(self, ncu: int) -> None:
        _check(load_library().piperag_set_compute_units(self._h, int(ncu)))

    def stage_times(self) -> np.ndarray:
        out = np.empty(NSTAGES, dtype=np.float32)
        _check(load_library().piperag_stage_times(self._h, out.ctypes.data))
        return out
