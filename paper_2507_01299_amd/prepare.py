"""Offline preparation of LaRoSA operands (not on the decode hot path): PCA rotations from
calibration tokens (Sec. 4.2), folding Q^T into the weights that meet a rotated input
(Sec. 4.3, Eq. 9-10), residual adapters Q_l^T Q_{l+1} (Sec. 4.2), one rounding to 16-bit
storage.  Plain fp64 torch linear algebra (library GEMM / eigensolver) on the device given.
"""
from __future__ import annotations

import torch

RMS_EPS = 1e-5


def _f64(a, device):
    return torch.as_tensor(a).to(device=device, dtype=torch.float64)


def rmsnorm(X: torch.Tensor, eps: float = RMS_EPS) -> torch.Tensor:
    return X / torch.sqrt((X * X).mean(dim=-1, keepdim=True) + eps)


def second_moment(X: torch.Tensor) -> torch.Tensor:
    """Averaged uncentred second moment of calibration tokens (rows of X), Sec. 4.2 Eq. 7."""
    return (X.T @ X) / X.shape[0]


def pca_rotation(C: torch.Tensor) -> torch.Tensor:
    """Eigenvectors of C as columns, eigenvalues descending (Sec. 4.2); column signs fixed so
    each column's largest-magnitude entry is positive.  The symmetric eigensolver runs on the
    host (LAPACK); its input and output live on C's device."""
    w, V = torch.linalg.eigh(C.cpu())
    order = torch.argsort(w, descending=True, stable=True)
    V = V[:, order]
    piv = V.abs().argmax(dim=0)
    sg = torch.sign(V[piv, torch.arange(V.shape[1])])
    sg[sg == 0] = 1.0
    return (V * sg[None, :]).to(C.device)


def fold_input_side(Q: torch.Tensor, W: torch.Tensor) -> torch.Tensor:
    """W' = Q^T W for W in the math layout [d_in, d_out]: row i of W' meets rotated channel i."""
    return Q.T @ W


def residual_adapter(Q_l: torch.Tensor, Q_next: torch.Tensor) -> torch.Tensor:
    return Q_l.T @ Q_next


def store(t: torch.Tensor, dtype: torch.dtype) -> torch.Tensor:
    return t.to(dtype).contiguous()


def gqa_repeat(v: torch.Tensor, d_q: int, d_kv: int, head_dim: int) -> torch.Tensor:
    g = (d_q // head_dim) // (d_kv // head_dim)
    return v.reshape(v.shape[0], d_kv // head_dim, head_dim).repeat_interleave(g, dim=1).reshape(v.shape[0], d_q)


def block_layer_operands(shape, W: dict, Xcal, dtype: torch.dtype, device, use_rms: bool = True) -> dict:
    """Operands of one decoder layer with explicit per-block rotations: Q_attn from the (normed)
    layer input, Q_mlp from the (normed) MLP-block input reached by pushing the calibration
    tokens through the dense attention half; q|k|v and gate|up folded on the input side."""
    X = _f64(Xcal, device)
    Wd = {k: _f64(v, device) for k, v in W.items()}
    N = rmsnorm(X) if use_rms else X
    Q_attn = pca_rotation(second_moment(N))
    a = gqa_repeat(N @ Wd["v"], shape.d_q, shape.d_kv, shape.head_dim)
    X1 = X + a @ Wd["o"]
    N1 = rmsnorm(X1) if use_rms else X1
    Q_mlp = pca_rotation(second_moment(N1))
    Wqkv = torch.cat([Wd["q"], Wd["k"], Wd["v"]], dim=1)
    Wgu = torch.cat([Wd["gate"], Wd["up"]], dim=1)
    return dict(
        Wqkv=store(fold_input_side(Q_attn, Wqkv), dtype), Wo=store(Wd["o"], dtype),
        Wgu=store(fold_input_side(Q_mlp, Wgu), dtype), Wdown=store(Wd["down"], dtype),
        Q_attn=store(Q_attn, dtype), Q_mlp=store(Q_mlp, dtype),
        # the same layer with every rotation absorbed (block-level form): o and down folded on the
        # output side, residual adapters on the two shortcuts; the layer after it is taken to use
        # the same attention basis, so its output is again a valid input
        Wo_out=store(Wd["o"] @ Q_mlp, dtype), Wdown_out=store(Wd["down"] @ Q_attn, dtype),
        shortcut_attn=store(residual_adapter(Q_attn, Q_mlp), dtype),
        shortcut_mlp=store(residual_adapter(Q_mlp, Q_attn), dtype))
