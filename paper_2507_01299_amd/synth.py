"""Seeded synthetic inputs for the LaRoSA decode path.

This module only draws random numbers and shapes them like the workloads the
paper measures (LLaMA-family projection shapes, low-rank-plus-outlier
activations).  It holds none of the method's arithmetic: no rotation, no PCA,
no Top-K, no folding, no 16-bit rounding.  Both the CPU oracle's tests and the
HIP path's tests/bench take their raw inputs from here so that they see the
same numbers.

Recipe (per token):  z ~ N(0, I_d)  (or Student-t, nu=3, per coordinate),
s_i = i^-0.8 (i = 1..d), U = sign-fixed Q-factor of a seeded d x d Gaussian,
x = (z * s) U^T, then four seeded distinct channels of x are multiplied by 20,
and a fixed scalar brings the expected RMS over channels to 1.
Weights are W ~ N(0, 0.02^2) in the math layout [d_in, d_out].
"""
from __future__ import annotations

import dataclasses
import numpy as np

BASE_SEED = 1299
RMS_EPS = 1e-5          # pre-norm epsilon of the synthetic layers (the paper gives none)


def seed_for(config: int, stream: int) -> int:
    """Sub-seed for (config, stream): 1299*1000 + 10*config + stream."""
    return BASE_SEED * 1000 + 10 * int(config) + int(stream)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def planted_basis(d: int, seed: int) -> np.ndarray:
    """Random orthogonal d x d matrix: Q-factor of a Gaussian, columns multiplied
    by sign(diag R) so the draw is unique (Haar distributed)."""
    g = _rng(seed).standard_normal((d, d))
    q, r = np.linalg.qr(g)
    sg = np.sign(np.diag(r))
    sg[sg == 0] = 1.0
    return q * sg[None, :]


def spectrum(d: int, power: float = 0.8) -> np.ndarray:
    return np.arange(1, d + 1, dtype=np.float64) ** (-power)


@dataclasses.dataclass
class ActivationSource:
    """A fixed distribution of tokens: planted basis, spectrum, outlier channels."""
    d: int
    U: np.ndarray            # [d, d] orthogonal
    s: np.ndarray            # [d]
    outliers: np.ndarray     # [n_out] int channel ids
    outlier_gain: float
    scale: float             # fixed scalar so that the expected RMS over channels is 1
    latent: str              # "gauss" | "t3"

    def draw(self, n: int, seed: int) -> np.ndarray:
        """n tokens, float64 [n, d]."""
        rng = _rng(seed)
        if self.latent == "gauss":
            z = rng.standard_normal((n, self.d))
        elif self.latent == "t3":
            # Student-t with 3 degrees of freedom, scaled to unit variance (var = nu/(nu-2) = 3)
            z = rng.standard_t(3.0, size=(n, self.d)) / np.sqrt(3.0)
        else:
            raise ValueError(self.latent)
        x = (z * self.s[None, :]) @ self.U.T
        x[:, self.outliers] *= self.outlier_gain
        return x * self.scale


def activation_source(d: int, seed: int, n_outliers: int = 4, outlier_gain: float = 20.0,
                      latent: str = "gauss", power: float = 0.8) -> ActivationSource:
    U = planted_basis(d, seed)
    s = spectrum(d, power)
    outliers = np.sort(_rng(seed + 1).choice(d, size=min(n_outliers, d), replace=False))
    # E[x_c^2] = sum_i s_i^2 U_ci^2, times gain^2 on outlier channels
    ex2 = (U * U) @ (s * s)
    ex2[outliers] *= outlier_gain ** 2
    scale = 1.0 / np.sqrt(ex2.mean())
    return ActivationSource(d, U, s, outliers, outlier_gain, float(scale), latent)


def gaussian_weight(d_in: int, d_out: int, seed: int, std: float = 0.02) -> np.ndarray:
    """W ~ N(0, std^2), math layout [d_in, d_out] (y = x W), float32 values."""
    return _rng(seed).standard_normal((d_in, d_out), dtype=np.float32) * np.float32(std)


@dataclasses.dataclass
class LayerShape:
    name: str
    d: int
    d_q: int
    d_kv: int
    d_ff: int
    head_dim: int
    dtype: str   # "f16" | "bf16"


SHAPES = {
    "tiny": LayerShape("tiny", 256, 256, 128, 704, 32, "f16"),
    "llama2-7b": LayerShape("llama2-7b", 4096, 4096, 4096, 11008, 128, "f16"),
    "llama3-8b": LayerShape("llama3-8b", 4096, 4096, 1024, 14336, 128, "bf16"),
    "llama2-70b": LayerShape("llama2-70b", 8192, 8192, 1024, 28672, 128, "bf16"),
}


def layer_weights(shape: LayerShape, seed: int) -> dict:
    """The seven projection matrices of one decoder layer, math layout [d_in, d_out]."""
    return {
        "q": gaussian_weight(shape.d, shape.d_q, seed + 0),
        "k": gaussian_weight(shape.d, shape.d_kv, seed + 1),
        "v": gaussian_weight(shape.d, shape.d_kv, seed + 2),
        "o": gaussian_weight(shape.d_q, shape.d, seed + 3),
        "gate": gaussian_weight(shape.d, shape.d_ff, seed + 4),
        "up": gaussian_weight(shape.d, shape.d_ff, seed + 5),
        "down": gaussian_weight(shape.d_ff, shape.d, seed + 6),
    }
