"""ctypes front end of the on-device workload generator (workload/gen_hip.hip).  Output is bit-identical
to `workload.gen.rows`."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np
import torch

from . import gen

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen_hip.hip")
_LIB = os.path.join(_HERE, "libworkload_hip.so")
_lib = None


def build() -> str:
    tmp = f"{_LIB}.{os.getpid()}.tmp"
    subprocess.check_call(["/opt/rocm/bin/hipcc", "-O3", "--offload-arch=gfx950", "-fPIC", "-shared", "-ffp-contract=off",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", tmp, _SRC])
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = C.CDLL(_LIB)
        _lib.workload_gen_rows.argtypes = [C.c_uint64, C.c_uint64, C.c_int64, C.c_int32, C.c_float, C.c_void_p, C.c_void_p,
                                           C.c_int32, C.c_void_p, C.c_void_p]
        _lib.workload_gen_rows.restype = C.c_int
        _lib.workload_plain_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        _lib.workload_plain_copy.restype = C.c_int
        _lib.workload_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        _lib.workload_stream_read.restype = C.c_int
    return _lib


class DeviceGenerator:
    """Holds the mixture tables of one configuration on the GPU."""

    def __init__(self, cfg: gen.WorkloadConfig, device: str = "cuda"):
        self.cfg = cfg
        self.centres = torch.from_numpy(gen.centres(cfg)).to(device)
        self.cum = torch.from_numpy(gen.component_cum(cfg).view(np.int64)).to(device)

    def rows(self, row0: int, count: int, out: torch.Tensor | None = None) -> torch.Tensor:
        cfg = self.cfg
        if out is None:
            out = torch.empty((count, cfg.d), dtype=torch.float32, device=self.centres.device)
        assert out.is_contiguous() and out.dtype == torch.float32 and out.numel() >= count * cfg.d
        rc = _load().workload_gen_rows(cfg.seed, row0, count, cfg.d, cfg.sigma, self.centres.data_ptr(), self.cum.data_ptr(),
                                       cfg.n_components, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise RuntimeError(f"workload_gen_rows failed with hipError {rc}")
        return out[:count] if out.shape[0] != count else out

    def database(self, start: int, count: int, out: torch.Tensor | None = None) -> torch.Tensor:
        assert 0 <= start and start + count <= self.cfg.N
        return self.rows(start, count, out)

    def queries(self, nq: int, start: int = 0) -> torch.Tensor:
        return self.rows(gen.QUERY_ROW0 + start, nq)


def plain_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    """Launches the plain copy kernel (profiling calibration: its HBM traffic is 2 * nbytes by construction)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and nbytes % 16 == 0
    rc = _load().workload_plain_copy(src.data_ptr(), dst.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"workload_plain_copy failed with hipError {rc}")


def stream_read(src: torch.Tensor, workgroups: int, nontemporal: bool, sink: torch.Tensor) -> None:
    """Launches the read-only reference kernel over src (roofline reference: nothing is computed or written)."""
    nbytes = src.numel() * src.element_size()
    rc = _load().workload_stream_read(src.data_ptr(), nbytes, int(workgroups), int(nontemporal), sink.data_ptr(),
                                      torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"workload_stream_read failed with hipError {rc}")
