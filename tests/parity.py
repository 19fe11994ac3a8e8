"""Tie-aware comparison of library results with the CPU oracle.

Tolerance: distances agree within 1e-4 relative (plus 1e-5 absolute, which only matters when the
distance itself is ~0, e.g. identity codebooks).  Integer results (list numbers, code bytes, ids)
must be identical unless the two alternatives are themselves within that tolerance in the oracle's
own arithmetic - only then may fp32 rounding order legitimately decide differently.
"""
from __future__ import annotations

import numpy as np

import oracle

RTOL = 1e-4
ATOL = 1e-5


def close(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.abs(a - b) <= RTOL * np.maximum(np.abs(a), np.abs(b)) + ATOL


def full_coarse_distances(q, coarse):
    """Oracle distance of every query to every centre, [nq, nlist] f32."""
    probes, dist = oracle.coarse_search(q, coarse, coarse.shape[0])
    full = np.empty_like(dist)
    np.put_along_axis(full, probes.astype(np.int64), dist, axis=1)
    return full


def check_probes(gpu_lists, gpu_dist, q, coarse, nprobe):
    """Returns the number of queries whose probe set differs from the oracle's (only allowed at ties)."""
    full = full_coarse_distances(q, coarse)
    o_probes, o_dist = oracle.coarse_search(q, coarse, nprobe)
    excused = 0
    for qi in range(q.shape[0]):
        g = gpu_lists[qi].astype(np.int64)
        assert len(set(g.tolist())) == nprobe, f"query {qi}: duplicate probe"
        assert g.min() >= 0 and g.max() < coarse.shape[0]
        if gpu_dist is not None:
            assert np.all(close(gpu_dist[qi], full[qi, g])), f"query {qi}: coarse distances off"
            assert np.all(np.diff(gpu_dist[qi]) >= 0), f"query {qi}: probes not sorted by distance"
        if np.array_equal(g, o_probes[qi]):
            continue
        tau = float(o_dist[qi, -1])
        # every chosen list is within tolerance of the cut, every list clearly inside the cut is chosen
        assert np.all(full[qi, g] <= tau * (1 + RTOL) + ATOL), f"query {qi}: probe beyond the cut"
        must = np.nonzero(full[qi] < tau * (1 - RTOL) - ATOL)[0]
        assert set(must.tolist()) <= set(g.tolist()), f"query {qi}: a clearly closer list was not probed"
        # order may differ only between lists whose distances are within tolerance
        assert np.all(close(np.sort(full[qi, g]), full[qi, g])), f"query {qi}: probe order off"
        excused += 1
    return excused


def check_topk(gpu_dist, gpu_ids, index: oracle.Index, q, probes, k):
    """Compares a top-k result with the oracle scanning the same probe lists.  Returns (number of
    queries whose id lists are not identical to the oracle's, max relative distance error)."""
    nq = q.shape[0]
    lens = np.diff(index.list_off)
    excused = 0
    max_rel = 0.0
    for qi in range(nq):
        pr = probes[qi:qi + 1]
        ncand = int(lens[pr[pr >= 0]].sum())
        search_fn = oracle.search_residual_with_probes if index.residual else oracle.search_with_probes
        scan_fn = oracle.scan_residual_with_probes if index.residual else oracle.scan_with_probes
        od, oi, scanned = search_fn(index, q[qi:qi + 1], pr, k)
        od, oi = od[0], oi[0]
        tau = od[min(k, ncand) - 1] if ncand > 0 else np.inf
        # every candidate the oracle places within tolerance of its k-th distance (any number of them may tie)
        ad, ai = scan_fn(index, q[qi], pr[0])
        near = ad <= tau * (1 + RTOL) + ATOL
        near_d, near_i = ad[near], ai[near]
        nvalid = min(k, ncand)
        gd, gi = gpu_dist[qi], gpu_ids[qi]
        assert np.all(gi[nvalid:] == -1) and np.all(np.isinf(gd[nvalid:])), f"query {qi}: padding wrong"
        gd, gi = gd[:nvalid], gi[:nvalid]
        assert len(set(gi.tolist())) == nvalid, f"query {qi}: duplicate ids"
        assert np.all(np.diff(gd) >= 0), f"query {qi}: distances not ascending"
        same_d = np.diff(gd) == 0
        assert np.all(np.diff(gi)[same_d] > 0), f"query {qi}: equal distances not ordered by id"
        omap = {int(i): float(d) for i, d in zip(near_i, near_d)}
        for i, d in zip(gi, gd):
            assert int(i) in omap, f"query {qi}: id {i} (dist {d}) is not among the oracle's candidates up to the cut"
            assert close(d, omap[int(i)]), f"query {qi}: id {i} distance {d} vs oracle {omap[int(i)]}"
            if omap[int(i)] > 0:
                max_rel = max(max_rel, abs(d - omap[int(i)]) / omap[int(i)])
            assert omap[int(i)] <= tau * (1 + RTOL) + ATOL, f"query {qi}: id {i} beyond the k-th distance"
        must = oi[:nvalid][od[:nvalid] < tau * (1 - RTOL) - ATOL]
        assert set(must.tolist()) <= set(gi.tolist()), f"query {qi}: a clearly closer vector is missing"
        if not np.array_equal(gi, oi[:nvalid]):
            excused += 1
    return excused, max_rel


def check_encoding(gpu_lists, gpu_codes, x, coarse, pq, residual=False):
    """List numbers and code bytes equal the oracle's, except where the oracle's own two distances are
    within tolerance.  Returns (list differences excused, code-byte differences excused).  residual: the codes
    quantise x minus the centre of its list; rows whose list differs (an excused tie) are then compared with the
    oracle's codes for the list the library chose."""
    o_lists, o_codes = oracle.encode(x, coarse, pq)
    M, ksub, dsub = pq.shape
    bad_l = np.nonzero(gpu_lists != o_lists)[0]
    for i in bad_l:
        d = oracle.coarse_search(x[i:i + 1], coarse[[o_lists[i], gpu_lists[i]]], 2)[1][0]
        assert close(d[0], d[1]), f"row {i}: list {gpu_lists[i]} vs oracle {o_lists[i]}, distances {d}"
    xq = x
    if residual:
        xq = oracle.residuals(x, coarse, gpu_lists)
        o_codes = oracle.encode(xq, coarse, pq)[1]
    bad_c = np.argwhere(gpu_codes != o_codes)
    if len(bad_c):
        for i, m in bad_c:
            table = oracle.lut(xq[i:i + 1], pq)[0, m]
            a, b = table[o_codes[i, m]], table[gpu_codes[i, m]]
            assert close(a, b), f"row {i} sub-quantiser {m}: code {gpu_codes[i, m]} vs oracle {o_codes[i, m]} ({b} vs {a})"
    return len(bad_l), len(bad_c)


def check_lists_screened(gpu_lists, x_dev, x_host, coarse, max_cand=64, block=16384):
    """List numbers of many rows against the oracle, at a cost that allows a million rows against 65,536 centres
    (the plain oracle does a few hundred such rows per second).  A library matrix product on the GPU (torch, fp32;
    harness code, not the library under test) first rules out the centres that are far from a row: those whose
    |c|^2 - 2<x, c> exceeds the row's smallest by more than a margin of 50 times the tolerance, taken relative to
    the distance, plus 1e-5 (|x|^2 + max |c|^2) for the product's own rounding.  The oracle (plain loops, fp64
    accumulation) then picks the nearest of the centres left, `oracle.assign_among`; rows with more than max_cand
    centres left go to the plain oracle over all centres.  Differences from the library's list numbers are excused
    exactly as in check_encoding: only if the oracle's own two distances are within tolerance.
    Returns (rows whose list differs, rows given to the plain oracle)."""
    import torch
    torch.backends.cuda.matmul.allow_tf32 = False
    n = x_host.shape[0]
    cd = torch.from_numpy(np.ascontiguousarray(coarse)).cuda()
    cn = (cd.double() ** 2).sum(1).float()
    cmax = float(cn.max())
    o_lists = np.empty(n, dtype=np.int32)
    n_full = 0
    for a in range(0, n, block):
        xb = x_dev[a:a + block]
        xn = (xb.double() ** 2).sum(1).float()
        v = cn[None, :] - 2.0 * (xb @ cd.T)
        best = v.min(dim=1).values
        margin = 50 * RTOL * torch.clamp(best + xn, min=0.0) + 1e-5 * (xn + cmax)
        mask = v <= (best + margin)[:, None]
        counts = mask.sum(1)
        few = counts <= max_cand
        cand = torch.full((xb.shape[0], max_cand), -1, dtype=torch.int32, device="cuda")
        rows, cols = torch.nonzero(mask & few[:, None], as_tuple=True)            # row-major order: runs of one row
        first = torch.zeros(xb.shape[0] + 1, dtype=torch.int64, device="cuda")
        first[1:] = torch.cumsum(torch.where(few, counts, torch.zeros_like(counts)), 0)
        cand[rows, (torch.arange(rows.shape[0], device="cuda") - first[rows]).long()] = cols.int()
        few_h, cand_h = few.cpu().numpy(), cand.cpu().numpy()
        xs = x_host[a:a + block]
        out = np.empty(xs.shape[0], dtype=np.int32)
        if few_h.any():
            out[few_h] = oracle.assign_among(xs[few_h], coarse, cand_h[few_h])
        if not few_h.all():
            out[~few_h] = oracle.assign(xs[~few_h], coarse)
            n_full += int((~few_h).sum())
        o_lists[a:a + block] = out
    bad = np.nonzero(gpu_lists != o_lists)[0]
    for i in bad:
        d = oracle.coarse_search(x_host[i:i + 1], coarse[[o_lists[i], gpu_lists[i]]], 2)[1][0]
        assert close(d[0], d[1]), f"row {i}: list {gpu_lists[i]} vs oracle {o_lists[i]}, distances {d}"
    return len(bad), n_full


def check_codes(gpu_codes, x_host, pq):
    """Code bytes against the plain oracle; differences only where the oracle's two table entries are within tolerance.
    Returns the number of differing bytes."""
    o_codes = oracle.encode_codes(x_host, pq)
    bad = np.argwhere(gpu_codes != o_codes)
    for i, m in bad:
        table = oracle.lut(x_host[i:i + 1], pq)[0, m]
        a, b = table[o_codes[i, m]], table[gpu_codes[i, m]]
        assert close(a, b), f"row {i} sub-quantiser {m}: code {gpu_codes[i, m]} vs oracle {o_codes[i, m]} ({b} vs {a})"
    return len(bad)
