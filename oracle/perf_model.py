"""CPU oracle of the paper's two performance models (test infrastructure: only tests/, the smoke entry and the
bench's CPU baseline may import this package; the product never does).

max_nprobe      - Section 3.2, S3: the retrieval latency is modelled as a line in nprobe; given the time T(C) the
                  next token chunk takes to generate, the largest search space whose predicted latency fits.
project_latency - Appendix "Performance Modeling for Future Hardware": sequential generation costs the sum of all
                  inference and retrieval times; pipelined generation costs inference + retrieval for the first
                  chunk and the larger of the two for every later chunk; either side may be scaled by a speed-up.

Plain Python on exact rationals (fractions.Fraction), so that no floating-point rounding enters the definition.
"""
from __future__ import annotations

from fractions import Fraction


def _frac(x) -> Fraction:
    return Fraction(float(x))            # the exact value of the binary floating-point number


def max_nprobe(fit, budget_ms, nprobe_cap: int, overhead_ms=0.0):
    """(nprobe, fits): by exhaustive search over 1..nprobe_cap, as the definition reads."""
    a, b, o, T = _frac(fit[0]), _frac(fit[1]), _frac(overhead_ms), _frac(budget_ms)
    best = None
    for p in range(1, nprobe_cap + 1):
        if o + a + b * p <= T:
            best = p if best is None else max(best, p)
    fits_one = o + a + b * 1 <= T
    if not fits_one:
        return 1, False
    if b <= 0:
        return nprobe_cap, True
    return best, True


def project_latency(inference_ms, retrieval_ms, inference_speedup=1.0, retrieval_speedup=1.0):
    """(sequential_ms, pipelined_ms) as exact rationals converted to float at the end."""
    si, sr = _frac(inference_speedup), _frac(retrieval_speedup)
    seq = Fraction(0)
    pipe = Fraction(0)
    for c, (ti, tr) in enumerate(zip(inference_ms, retrieval_ms)):
        ti, tr = _frac(ti) / si, _frac(tr) / sr
        seq += ti + tr
        pipe += ti + tr if c == 0 else max(ti, tr)
    return float(seq), float(pipe)
