"""Oracle of the heterogeneous-aware allocation.  TEST INFRASTRUCTURE ONLY.

HEXA-MoE Sec. 3.4: device i, whose measured latency on a common benchmark task is t_i, gets
the share (1/t_i) / sum_j (1/t_j) of the work: of the global batch size (Eq. 1, data-centric) or
of the FFN hidden size (Eq. 2, model-centric).  The paper then asks for the shares to be rounded
"up or down" so that they are integers with an exact sum and leaves the rule open.  The reading
taken here (and by the library): largest-remainder rounding in units of `granule`; every device
gets the floor of its ideal share and the units left over go one each to the largest fractional
parts, equal fractions to the lower device index.

Everything is exact rational arithmetic (a double converts to a Fraction without rounding), in
the order of the formulas; no part of the library is imported.  Pins
(tests/test_oracle_pins.py): the capacity proportions the paper prints for its two-GPU machine
(Sec. 4 Table 2, stored in tests/golden/), equal latencies, exact sums, and a brute force over
all integer splits on tiny inputs.  Only tests may import this module.
"""
from fractions import Fraction
from typing import List, Sequence


def ideal_shares(latency: Sequence[float], total: int) -> List[Fraction]:
    """Eq. 1 / Eq. 2 before rounding: total * (1/t_i) / sum_j (1/t_j), exactly."""
    if len(latency) == 0 or any(not (t > 0) for t in latency):
        raise ValueError("latencies must be positive")
    inv = [Fraction(1) / Fraction(t) for t in latency]
    s = sum(inv)
    return [w / s * total for w in inv]


def allocate(latency: Sequence[float], total: int, granule: int = 1) -> List[int]:
    """Integer shares (multiples of granule, summing to total) by largest remainders."""
    if granule < 1 or total < 0 or total % granule != 0:
        raise ValueError("total must be a non-negative multiple of granule >= 1")
    units = total // granule
    ideal = ideal_shares(latency, units)
    share = [int(q) for q in ideal]               # floor: every q is >= 0
    frac = [q - s for q, s in zip(ideal, share)]
    left = units - sum(share)
    order = sorted(range(len(latency)), key=lambda i: (-frac[i], i))
    for i in order[:left]:
        share[i] += 1
    return [s * granule for s in share]
