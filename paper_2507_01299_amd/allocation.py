"""Kept counts per activation type (App. B of the paper): k_i = alpha_i (1 - p) D_i for h1..h4 with
alpha_2 and alpha_4 tied to alpha_1 and alpha_3 by the block constraints 3 alpha_1 + alpha_2 = 4
(attention block) and 2 alpha_3 + M alpha_4 = 2 + M (MLP block, M = d_ff / d), so that the number of kept
activation entries per block stays what uniform alpha = 1 gives.  Host-side bookkeeping only: the
kernels take K1..K4.

The arithmetic is exact: sparsity and coefficients are decimal numbers as a user types them (0.4, 0.90),
and k = alpha (1 - p) D sits on or next to an integer for the usual widths (0.75 * 4096 = 3072), where
binary floating point would decide the truncation by its rounding error."""
from __future__ import annotations

from fractions import Fraction


def _exact(x) -> Fraction:
    """The decimal number the caller wrote: 0.4 -> 2/5 (not the nearest binary64)."""
    return x if isinstance(x, Fraction) else Fraction(str(x))


def kept_counts(d: int, d_q: int, d_ff: int, p, alpha1=1, alpha3=1):
    """(K1, K2, K3, K4) for h1 (width d), h2 (d_q), h3 (d), h4 (d_ff): the integer part of
    alpha_i (1 - p) D_i, at least 1 and at most the width."""
    keep = 1 - _exact(p)
    a1, a3 = _exact(alpha1), _exact(alpha3)
    M = Fraction(d_ff, d)
    a2 = 4 - 3 * a1                      # 3 alpha_1 + alpha_2 = 4
    a4 = (2 + M - 2 * a3) / M            # 2 alpha_3 + M alpha_4 = 2 + M
    return tuple(min(width, max(1, (a * keep * width).__floor__()))
                 for a, width in ((a1, d), (a2, d_q), (a3, d), (a4, d_ff)))


def selected_weight_bytes(d: int, d_q: int, d_kv: int, d_ff: int, Ks, elem_bytes: int = 2) -> int:
    """Bytes of weight rows one token reads in a layer: K1 rows of q|k|v, K2 of o, K3 of gate|up, K4 of down."""
    K1, K2, K3, K4 = Ks
    return elem_bytes * (K1 * (d_q + 2 * d_kv) + K2 * d + K3 * 2 * d_ff + K4 * d)
