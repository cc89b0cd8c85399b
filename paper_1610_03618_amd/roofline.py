"""Algorithmic byte counts for the roofline: what each operation must move.

Every needed input element is read once and every output element written once,
fp32 (4 bytes).  Used by the benchmark and by the bandwidth reports only.
"""
from __future__ import annotations

PEAK_HBM_GBPS = 8000.0   # MI355X published HBM3E peak


def pooled_extent(L: int, k: int, s: int, p: int) -> int:
    return (L + 2 * p - k) // s + 1


def transform_bytes(N: int, C: int, H: int, W: int) -> int:
    return 2 * 4 * N * C * H * W


def pool_bytes(N: int, C: int, H: int, W: int, kh: int, kw: int, sh: int, sw: int,
               ph: int = 0, pw: int = 0) -> int:
    Ho, Wo = pooled_extent(H, kh, sh, ph), pooled_extent(W, kw, sw, pw)
    Hc = min(H, (Ho - 1) * sh + kh - ph)   # input rows some window covers
    Wc = min(W, (Wo - 1) * sw + kw - pw)
    return 4 * N * C * (Hc * Wc + Ho * Wo)


def softmax_bytes(N: int, classes: int) -> int:
    return 2 * 4 * N * classes


def pool_backward_bytes(N: int, C: int, H: int, W: int, kh: int, kw: int, sh: int, sw: int,
                        ph: int = 0, pw: int = 0, needs_input: bool = True) -> int:
    """Read the incoming gradient (and, for the maximum, the forward input), write every input gradient."""
    Ho, Wo = pooled_extent(H, kh, sh, ph), pooled_extent(W, kw, sw, pw)
    Hc = min(H, (Ho - 1) * sh + kh - ph)
    Wc = min(W, (Wo - 1) * sw + kw - pw)
    return 4 * N * C * (H * W + Ho * Wo + (Hc * Wc if needs_input else 0))


def softmax_backward_bytes(N: int, classes: int) -> int:
    return 3 * 4 * N * classes
