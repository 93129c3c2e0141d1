"""Kept counts per activation type (App. B of the paper): k_i = alpha_i (1 - p) D_i for h1..h4 with
alpha_2 = 4 - 3 alpha_1 (attention block) and alpha_4 = (2 + M - 2 alpha_3) / M (MLP block,
M = d_ff / d), so that the number of kept activation entries per block stays what uniform
alpha = 1 gives.  Host-side bookkeeping only: the kernels take K1..K4."""
from __future__ import annotations

import math


def _count(alpha: float, p: float, width: int) -> int:
    return max(1, min(int(width), int(math.floor(alpha * (1.0 - p) * width + 1e-9))))


def kept_counts(d: int, d_q: int, d_ff: int, p: float, alpha1: float = 1.0, alpha3: float = 1.0):
    """(K1, K2, K3, K4) for h1 (width d), h2 (d_q), h3 (d), h4 (d_ff); counts are clamped to the width."""
    M = d_ff / d
    alpha2 = 4.0 - 3.0 * alpha1
    alpha4 = (2.0 + M - 2.0 * alpha3) / M
    return (_count(alpha1, p, d), _count(alpha2, p, d_q), _count(alpha3, p, d), _count(alpha4, p, d_ff))


def selected_weight_bytes(d: int, d_q: int, d_kv: int, d_ff: int, Ks, elem_bytes: int = 2) -> int:
    """Bytes of weight rows one token reads in a layer: K1 rows of q|k|v, K2 of o, K3 of gate|up, K4 of down."""
    K1, K2, K3, K4 = Ks
    return elem_bytes * (K1 * (d_q + 2 * d_kv) + K2 * d + K3 * 2 * d_ff + K4 * d)
