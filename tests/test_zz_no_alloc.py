"""The entry point for callers that cannot allocate (piperag_ivfpq_search_static) against the ordinary search entry
point: same index, same queries, outputs equal bit for bit, on two calls in a row, the second smaller than the
first (the static scratch array keeps the first call's contents, laid out for the first call's sizes)."""
import ctypes

import numpy as np
import pytest

import oracle
import parity
from workload import gen

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def build_index(pkg, seed=77, N=120_000, d=64, nlist=300, M=16, nq=24):
    cfg = gen.WorkloadConfig(f"na{seed}", seed, 24, 1.0, 0.3, N, d, nlist, M, 20000, nq, 1, 1)
    x, q = gen.database(cfg), gen.queries(cfg, nq)
    ci = gen.draw_distinct_rows(20000, nlist, seed)
    pi = [gen.draw_distinct_rows(20000, 256, seed + 1 + m) for m in range(M)]
    coarse, pq = oracle.train(x[:20000], nlist, M, ci, pi, iters=3)
    oidx = oracle.make_index(x, coarse, pq)
    # limits far below what the static entry point is asked for: it must not depend on them
    ix = pkg.Index.ivf_create(coarse, pq, N, max_nq=32, max_nprobe=64, max_k=64)
    lists = np.repeat(np.arange(nlist, dtype=np.int32), np.diff(oidx.list_off))
    ix.ivf_add_encoded(dev(lists), dev(oidx.codes), dev(oidx.ids))
    ix.ivf_finalize()
    return ix, oidx, q


def search_static_raw(pkg, ix, qd, nprobe, k):
    """Through the C ABI itself: raw pointers and sizes, the caller's buffers."""
    lib = pkg.load_library()
    nq = qd.shape[0]
    od = torch.full((nq, k), -7.0, dtype=torch.float32, device="cuda")
    oi = torch.full((nq, k), -7, dtype=torch.int64, device="cuda")
    rc = lib.piperag_ivfpq_search_static(ix._h, ctypes.c_void_p(qd.data_ptr()), nq, nprobe, k, ctypes.c_void_p(od.data_ptr()),
                                         ctypes.c_void_p(oi.data_ptr()), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return rc, od, oi


def test_static_scratch_search_equals_the_ordinary_search_twice_in_a_row():
    import paper_2403_05676_amd as pkg
    pkg.load_library()
    ix, oidx, q = build_index(pkg)
    qd = dev(q)
    for nq, nprobe, k in [(24, 48, 60), (5, 7, 9)]:           # the second call is smaller in every size
        sub = qd[:nq].contiguous()
        rd, ri = ix.ivfpq_search(sub, nprobe, k)
        torch.cuda.synchronize()
        want_scanned = ix.search_stats()
        rc, od, oi = search_static_raw(pkg, ix, sub, nprobe, k)
        assert rc == 0, pkg.load_library().piperag_last_error()
        torch.cuda.synchronize()
        assert torch.equal(od, rd), f"distances differ (nq={nq}, nprobe={nprobe}, k={k})"
        assert torch.equal(oi, ri), f"ids differ (nq={nq}, nprobe={nprobe}, k={k})"
        assert ix.search_stats() == want_scanned
        # and both agree with the oracle
        gl, _ = ix.ivf_coarse(sub, nprobe)
        torch.cuda.synchronize()
        ex, rel = parity.check_topk(od.cpu().numpy(), oi.cpu().numpy(), oidx, q[:nq], gl.cpu().numpy(), k)
        assert rel < 1e-4
    # a call beyond the index's own limits is fine (the static scratch does not depend on them) ...
    rc, od, oi = search_static_raw(pkg, ix, qd, 100, 128)
    assert rc == 0
    torch.cuda.synchronize()
    gl = oracle.coarse_search(q, oidx.coarse, 100)[0]
    ex, rel = parity.check_topk(od.cpu().numpy(), oi.cpu().numpy(), oidx, q, gl, 128)
    assert rel < 1e-4
    # ... and one beyond the scratch array is refused with a clear error, before anything is launched
    big = torch.zeros((60000, qd.shape[1]), dtype=torch.float32, device="cuda")
    rc, _, _ = search_static_raw(pkg, ix, big, 8, 4)
    assert rc == -5 and b"scratch" in pkg.load_library().piperag_last_error()
    # the ordinary entry point still works afterwards
    rd2, ri2 = ix.ivfpq_search(qd[:5].contiguous(), 7, 9)
    torch.cuda.synchronize()
    assert torch.equal(rd2, rd) and torch.equal(ri2, ri)
