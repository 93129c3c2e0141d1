"""The offline part of the method driven through the HIP library (Sec. 4.2): second moments of
calibration tokens, weight folding and residual adapters run on the matrix cores
(larosa_second_moment, larosa_fold_input, larosa_fold_output, larosa_residual_adapter); the
symmetric eigen-solver in between is a library call (torch.linalg.eigh in fp64).  Pushing the
calibration tokens through the dense model to reach a block's input is the model's own forward
pass, done here with plain torch matmuls.  Not on the decode hot path."""
from __future__ import annotations

import torch

from . import api


def _tname(t: torch.Tensor) -> str:
    return "f16" if t.dtype == torch.float16 else "bf16"


def rmsnorm16(X: torch.Tensor, eps: float) -> torch.Tensor:
    """Pre-norm of 16-bit calibration tokens, computed in fp32 and stored back in 16 bits (what the
    rotated projections of the deployed model will see)."""
    x = X.float()
    return (x * torch.rsqrt((x * x).mean(dim=-1, keepdim=True) + eps)).to(X.dtype)


def second_moment(X: torch.Tensor, batch: int = 8192) -> torch.Tensor:
    """Sum of x^T x over the rows of X [n, d] (16-bit), fp32 [d, d], fed in batches."""
    n, d = X.shape
    C = torch.empty(d, d, dtype=torch.float32, device=X.device)
    for i, s in enumerate(range(0, n, batch)):
        api.second_moment(X[s:s + batch].contiguous(), C, _tname(X), accumulate=i > 0)
    return C


def pca_rotation(C: torch.Tensor, solver_device=None) -> torch.Tensor:
    """Rotation Q of Sec. 4.2: the eigenvectors of the symmetric second moment C as columns, leading
    principal direction first.  The fp64 symmetric eigen-solver (a library call, on `solver_device`,
    default C's device) returns the spectrum ascending, so the columns are simply reversed; the result is
    fp32 on C's device.  A column's sign is whatever the solver returns: nothing downstream depends on
    it (h_i and row i of Q^T W change sign together, and the Top-K compares |h_i|)."""
    dev = C.device if solver_device is None else solver_device
    _, V = torch.linalg.eigh(C.to(device=dev, dtype=torch.float64))
    return torch.flip(V, dims=(1,)).to(device=C.device, dtype=torch.float32).contiguous()


def _gqa_repeat(v, d_q, d_kv, head_dim):
    g = (d_q // head_dim) // (d_kv // head_dim)
    return v.reshape(v.shape[0], d_kv // head_dim, head_dim).repeat_interleave(g, dim=1).reshape(v.shape[0], d_q)


def prepare_block_layer(shape, W: dict, Xcal: torch.Tensor, rms_eps: float = 1e-5, solver_device=None) -> dict:
    """Operands of one decoder layer with explicit per-block rotations.  W holds the dense 16-bit
    device weights q, k, v, o, gate, up, down in the [d_in, d_out] layout; Xcal [n, d] are 16-bit
    calibration tokens at the layer input.  Q_attn comes from the normed layer input, Q_mlp from the
    normed MLP-block input reached through the dense attention half (context length 1)."""
    t = _tname(Xcal)
    d = shape.d
    scratch = api.OfflineScratch(d, t)
    N = rmsnorm16(Xcal, rms_eps)
    Q_attn = pca_rotation(second_moment(N), solver_device)
    a = _gqa_repeat(N @ W["v"], shape.d_q, shape.d_kv, shape.head_dim)
    X1 = (Xcal.float() + (a @ W["o"]).float()).to(Xcal.dtype)
    Q_mlp = pca_rotation(second_moment(rmsnorm16(X1, rms_eps)), solver_device)
    Wqkv = torch.cat([W["q"], W["k"], W["v"]], dim=1).contiguous()
    Wgu = torch.cat([W["gate"], W["up"]], dim=1).contiguous()
    out = dict(Wqkv=torch.empty_like(Wqkv), Wgu=torch.empty_like(Wgu), Wo=W["o"].contiguous(),
               Wdown=W["down"].contiguous(), Q_attn=Q_attn.to(Xcal.dtype), Q_mlp=Q_mlp.to(Xcal.dtype),
               Q_attn32=Q_attn, Q_mlp32=Q_mlp)
    api.fold_input(Q_attn, Wqkv, out["Wqkv"], t, scratch)
    api.fold_input(Q_mlp, Wgu, out["Wgu"], t, scratch)
    torch.cuda.synchronize()
    return out


def prepare_shortcut_layer(shape, W: dict, Xcal: torch.Tensor, rms_eps: float = 1e-5, solver_device=None) -> dict:
    """The same layer with every rotation absorbed (the block-level form of Sec. 5.4 as it is deployed):
    on top of prepare_block_layer's operands, o carries Q_mlp and down carries Q_attn on the output side
    (Wo_out, Wdown_out: the layer after this one is taken to use the same attention basis, so its output
    is again a valid input), and the two shortcuts carry the residual adapters Q_attn^T Q_mlp
    (shortcut_attn) and Q_mlp^T Q_attn (shortcut_mlp) of Sec. 4.2.  The layer input then lives in the
    basis Q_attn."""
    t = _tname(Xcal)
    out = prepare_block_layer(shape, W, Xcal, rms_eps, solver_device)
    scratch = api.OfflineScratch(shape.d, t)
    Qa, Qm = out["Q_attn32"], out["Q_mlp32"]
    out["Wo_out"] = torch.empty_like(out["Wo"])
    out["Wdown_out"] = torch.empty_like(out["Wdown"])
    out["shortcut_attn"] = torch.empty(shape.d, shape.d, dtype=Xcal.dtype, device=Xcal.device)
    out["shortcut_mlp"] = torch.empty(shape.d, shape.d, dtype=Xcal.dtype, device=Xcal.device)
    api.fold_output(out["Wo"], Qm, out["Wo_out"], t, scratch)
    api.fold_output(out["Wdown"], Qa, out["Wdown_out"], t, scratch)
    api.residual_adapter(Qa, Qm, out["shortcut_attn"], t, scratch)
    api.residual_adapter(Qm, Qa, out["shortcut_mlp"], t, scratch)
    torch.cuda.synchronize()
    return out


def prepare_folded_layer(shape, W: dict, Q: torch.Tensor, Q_next: torch.Tensor) -> dict:
    """Operands of one decoder layer in the deployed form: the residual stream lives in the basis Q
    (fp32 [d, d]); q|k|v and gate|up carry Q^T on the input side, o and down carry Q on the output
    side, and the adapter Q^T Q_next takes the stream to the next layer's basis."""
    t = _tname(W["q"])
    scratch = api.OfflineScratch(shape.d, t)
    Wqkv = torch.cat([W["q"], W["k"], W["v"]], dim=1).contiguous()
    Wgu = torch.cat([W["gate"], W["up"]], dim=1).contiguous()
    out = dict(Wqkv=torch.empty_like(Wqkv), Wgu=torch.empty_like(Wgu), Wo=torch.empty_like(W["o"]),
               Wdown=torch.empty_like(W["down"]),
               adapter=torch.empty(shape.d, shape.d, dtype=W["q"].dtype, device=W["q"].device))
    api.fold_input(Q, Wqkv, out["Wqkv"], t, scratch)
    api.fold_input(Q, Wgu, out["Wgu"], t, scratch)
    api.fold_output(W["o"].contiguous(), Q, out["Wo"], t, scratch)
    api.fold_output(W["down"].contiguous(), Q, out["Wdown"], t, scratch)
    api.residual_adapter(Q, Q_next, out["adapter"], t, scratch)
    torch.cuda.synchronize()
    return out
