"""Caller-side problem set-up: the integers the C ABI takes, from the ratios the paper states.

The library's boundary carries the sparse count k and the Tucker ranks r_n as integers (computed
"by the caller, exactly").  A training script that starts from the paper's hyper-parameters - a
sparsity rho and a rank ratio per mode - uses these two helpers to get them; nothing in the
binding or in the kernels calls them.
"""
from __future__ import annotations

from fractions import Fraction


def sparse_count(density: Fraction, numel: int) -> int:
    """k = ceil(rho I) in exact integer arithmetic (section "Unstructured sparse gradient tensor")."""
    d = Fraction(density)
    q, r = divmod(d.numerator * int(numel), d.denominator)
    return int(q + (1 if r else 0))


def rank_from_ratio(ratio: Fraction, extent: int) -> int:
    """Round-half-up rank for a per-mode ratio, at least 1."""
    ratio = Fraction(ratio)
    return max(1, int((2 * ratio.numerator * extent + ratio.denominator) // (2 * ratio.denominator)))
