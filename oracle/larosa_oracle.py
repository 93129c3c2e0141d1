"""CPU fp64 oracle for the LaRoSA decode path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct numpy/fp64 statements of what the paper's method
computes, used to check the HIP kernels.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import this package; the product path never
does, and this file imports nothing from the product.

Every function cites the passage of the paper (arXiv 2507.01299) it follows.
16-bit tensors are carried as numpy uint16 bit patterns plus a dtype tag
("f16" | "bf16"); all arithmetic is fp64.

Pinned by tests/test_oracle_*.py (4-bit weights and the threshold sparsifier in
tests/test_oracle_w4_threshold.py) against closed forms, invariants, brute force
on tiny inputs and the values the paper prints (tests/golden/).  Unpinned:
nothing in this file.  (The paper's accuracy tables need real model weights
and datasets and are outside what this oracle states: parity unpinned there.)
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------
# 16-bit storage formats (IEEE binary16 and bfloat16), round-to-nearest-even
# --------------------------------------------------------------------------


def decode16(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Widen stored 16-bit patterns exactly to fp64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def _f64_to_f32_round_to_odd(v: np.ndarray) -> np.ndarray:
    """fp64 -> fp32 with round-to-odd (sticky LSB), so that a later RNE to a
    format with >= 2 fewer mantissa bits equals a single RNE from fp64."""
    v = np.asarray(v, dtype=np.float64)
    with np.errstate(over="ignore"):
        t = v.astype(np.float32)
    back = t.astype(np.float64)
    inexact = (back != v) & np.isfinite(v)
    # move to the neighbour toward zero when RNE went away from zero
    away = inexact & (np.abs(back) > np.abs(v))
    t = np.where(away, np.nextafter(t, np.float32(0.0)), t).astype(np.float32)
    b = t.view(np.uint32).copy()
    b[inexact] |= np.uint32(1)
    return b.view(np.float32)


def encode16(v: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to the 16-bit storage format (RNE), return uint16 bits."""
    v = np.asarray(v, dtype=np.float64)
    if dtype == "f16":
        with np.errstate(over="ignore"):
            return v.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        f = _f64_to_f32_round_to_odd(v)
        b = f.view(np.uint32).astype(np.uint64)
        lsb = (b >> np.uint64(16)) & np.uint64(1)
        r = ((b + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)
        nan = np.isnan(v)
        if np.any(nan):
            r = np.where(nan, np.uint16(0x7FC0), r).astype(np.uint16)
        return r
    raise ValueError(dtype)


def round16(v: np.ndarray, dtype) -> np.ndarray:
    """Value after one storage rounding (fp64 in, fp64 out).  dtype None = no rounding."""
    if dtype is None:
        return np.asarray(v, dtype=np.float64)
    return decode16(encode16(v, dtype), dtype)


# --------------------------------------------------------------------------
# Offline part: PCA rotation, folding, adapters  (Sec. 4.2, Sec. 3.2)
# --------------------------------------------------------------------------


def second_moment(X: np.ndarray) -> np.ndarray:
    """Averaged uncentred second-moment matrix of calibration tokens (Sec. 4.2, Eq. 7):
    C = (1/n) sum_t x_t^T x_t  with tokens as rows of X [n, d].  D x D."""
    X = np.asarray(X, dtype=np.float64)
    return (X.T @ X) / X.shape[0]


def pca_rotation(C: np.ndarray):
    """Q_l = eigenvectors of C as columns, eigenvalues in descending order (Sec. 4.2).
    Column i of Q is the i-th principal direction (App. A: x~_i = sum_j x_j Q_ji).
    Each column's sign is fixed so that its largest-magnitude entry is positive
    (outputs do not depend on the sign; this only makes Q reproducible).
    Returns (Q, eigenvalues)."""
    w, V = np.linalg.eigh(np.asarray(C, dtype=np.float64))
    order = np.argsort(-w, kind="stable")
    w = w[order]
    V = V[:, order]
    piv = np.argmax(np.abs(V), axis=0)
    sg = np.sign(V[piv, np.arange(V.shape[1])])
    sg[sg == 0] = 1.0
    return V * sg[None, :], w


def fold_input_side(Q: np.ndarray, W: np.ndarray) -> np.ndarray:
    """W' = Q^T W for W in the math layout [d_in, d_out] (Eq. 9-10: (W_pt Q)^T = Q^T W_pt^T).
    Row i of W' is the weight row met by rotated channel i."""
    return np.asarray(Q, np.float64).T @ np.asarray(W, np.float64)


def fold_output_side(W: np.ndarray, Q: np.ndarray) -> np.ndarray:
    """W Q: the producing projection emits its output already rotated (Sec. 3.2)."""
    return np.asarray(W, np.float64) @ np.asarray(Q, np.float64)


def residual_adapter(Q_l: np.ndarray, Q_next: np.ndarray) -> np.ndarray:
    """Q_l^T Q_{l+1}: takes the residual stream from layer l's basis to layer l+1's (Sec. 4.2)."""
    return np.asarray(Q_l, np.float64).T @ np.asarray(Q_next, np.float64)


def kept_count(d_in: int, p: float, alpha: float = 1.0) -> int:
    """k = alpha (1-p) D_in (Sec. 4.3), truncated to an integer, clamped to [1, D_in]."""
    k = int(np.floor(alpha * (1.0 - p) * d_in + 1e-9))
    return max(1, min(int(d_in), k))


def alpha_partner_attn(alpha1: float) -> float:
    """alpha_2 from alpha_1 under 3 alpha_1 + alpha_2 = 4 (App. B)."""
    return 4.0 - 3.0 * alpha1


def alpha_partner_mlp(alpha3: float, M: float) -> float:
    """alpha_4 from alpha_3 under 2 alpha_3 + M alpha_4 = 2 + M (App. B)."""
    return (2.0 + M - 2.0 * alpha3) / M


# --------------------------------------------------------------------------
# Online part: rotate, Top-K sparsifier, column-sparse projection (Sec. 4.3)
# --------------------------------------------------------------------------


def rotate(x: np.ndarray, Q: np.ndarray) -> np.ndarray:
    """h = x Q, i.e. h_i = sum_j x_j Q_ji (Sec. 4.3; App. A fixes the index convention).
    x [..., d] fp64, Q [d, d] fp64."""
    return np.asarray(x, np.float64) @ np.asarray(Q, np.float64)


def rmsnorm(x: np.ndarray, eps: float, scale=None) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) (* scale): the pre-norm in front of each block (Sec. 3.1-3.2)."""
    x = np.asarray(x, np.float64)
    r = x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return r if scale is None else r * np.asarray(scale, np.float64)


def magnitude_key(bits: np.ndarray) -> np.ndarray:
    """Ordering key of |h_i| on the stored 16-bit value: the bit pattern with the sign
    cleared, read as an unsigned integer.  Monotone in |h| for finite values,
    -0 == +0, Inf above finite, NaN patterns above Inf."""
    return (np.asarray(bits, dtype=np.uint16) & np.uint16(0x7FFF)).astype(np.int64)


def topk_indices(bits_row: np.ndarray, K: int) -> np.ndarray:
    """Indices kept by S_k (Eq. 8) for one token: the K entries of largest |h|,
    ties broken by larger magnitude first and then lower index; returned ascending.
    Stated as a full stable sort."""
    key = magnitude_key(bits_row)
    d = key.shape[0]
    if not (1 <= K <= d):
        raise ValueError("K out of range")
    order = np.argsort(-key, kind="stable")          # stable => lower index first among equals
    return np.sort(order[:K]).astype(np.int32)


def topk_batch(bits: np.ndarray, K: int) -> np.ndarray:
    bits = np.asarray(bits, dtype=np.uint16)
    return np.stack([topk_indices(r, K) for r in bits.reshape(-1, bits.shape[-1])]).reshape(
        bits.shape[:-1] + (K,))


def sparsify(h: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """S_k(h) (Eq. 8): h on the kept indices, 0 elsewhere.  One token."""
    out = np.zeros_like(np.asarray(h, np.float64))
    out[idx] = h[idx]
    return out


def sparse_project_gather(h: np.ndarray, idx: np.ndarray, Wp: np.ndarray) -> np.ndarray:
    """y_o = sum_t h[idx_t] W'[idx_t, o] (Eq. 10), one token; only the kept rows are read."""
    h = np.asarray(h, np.float64)
    return h[idx] @ np.asarray(Wp)[idx].astype(np.float64)


def sparse_project_masked(h: np.ndarray, idx: np.ndarray, Wp: np.ndarray) -> np.ndarray:
    """The same product written as S_k(h) W' over all rows (Eq. 10 with the mask explicit)."""
    return sparsify(h, idx) @ np.asarray(Wp, np.float64)


def sparse_project_batch(h: np.ndarray, idx: np.ndarray, Wp64: np.ndarray) -> np.ndarray:
    """Per-token index sets: y[b] = sum_t h[b, idx[b,t]] W'[idx[b,t], :]."""
    return np.stack([sparse_project_gather(h[b], idx[b], Wp64) for b in range(h.shape[0])])


# --------------------------------------------------------------------------
# 4-bit weights (W4A16, Sec. 5.4 / Table 9 use round-to-nearest codes; the paper
# fixes no storage format: groups of 128 output columns per input-channel row and
# the nibble order are this build's choice)
# --------------------------------------------------------------------------

W4_GROUP = 128


def quantize_rtn_w4(W: np.ndarray, dtype: str, group: int = W4_GROUP):
    """Symmetric round-to-nearest 4-bit codes of W [d_in, d_out], one scale per row and per
    group of `group` consecutive output columns: s = max|w| / 7 stored in 16 bits,
    q = clip(rint(w / s), -8, 7) + 8 in [0, 15] (q = 8 where s = 0).
    Returns (codes uint8 [d_in, d_out], scale bit patterns uint16 [d_in, ceil(d_out/group)])."""
    W = np.asarray(W, np.float64)
    d_in, d_out = W.shape
    ng = -(-d_out // group)
    codes = np.empty((d_in, d_out), np.uint8)
    sbits = np.empty((d_in, ng), np.uint16)
    for g in range(ng):
        blk = W[:, g * group:(g + 1) * group]
        sb = encode16(np.abs(blk).max(axis=1) / 7.0, dtype)
        s = decode16(sb, dtype)
        q = np.zeros_like(blk)
        nz = s > 0
        q[nz] = np.rint(blk[nz] / s[nz, None])
        codes[:, g * group:(g + 1) * group] = (np.clip(q, -8, 7) + 8).astype(np.uint8)
        sbits[:, g] = sb
    return codes, sbits


def dequantize_w4(codes: np.ndarray, sbits: np.ndarray, dtype: str, group: int = W4_GROUP) -> np.ndarray:
    """w = (q - 8) * s of the column's group, fp64."""
    s = decode16(sbits, dtype)
    cols = np.arange(codes.shape[1]) // group
    return (codes.astype(np.float64) - 8.0) * s[:, cols]


def pack_w4(codes: np.ndarray) -> np.ndarray:
    """Eight codes per little-endian dword: nibble k (bits 4k..4k+3) of dword m of a row is the
    code of column 8m + k.  [d_in, d_out] -> uint32 [d_in, d_out/8]."""
    c = np.asarray(codes, np.uint32).reshape(codes.shape[0], -1, 8)
    out = np.zeros(c.shape[:2], np.uint32)
    for k in range(8):
        out |= c[:, :, k] << np.uint32(4 * k)
    return out


def unpack_w4(packed: np.ndarray) -> np.ndarray:
    p = np.asarray(packed, np.uint32)
    return np.stack([(p >> np.uint32(4 * k)) & np.uint32(15) for k in range(8)], axis=-1).reshape(
        p.shape[0], -1).astype(np.uint8)


def sparse_project_w4(h: np.ndarray, idx: np.ndarray, codes: np.ndarray, sbits: np.ndarray, dtype: str) -> np.ndarray:
    """Eq. 10 over the dequantised 4-bit weight: y_o = sum_t h[idx_t] (q[idx_t,o] - 8) s[idx_t, g(o)]."""
    return np.asarray(h, np.float64)[idx] @ dequantize_w4(codes[idx], sbits[idx], dtype)


# --------------------------------------------------------------------------
# Magnitude-threshold sparsifier S_eps (Eq. 4-5): the comparison method whose kept
# count varies from token to token (Sec. 4.1)
# --------------------------------------------------------------------------


def calibrate_threshold(H: np.ndarray, p: float) -> float:
    """Cutoff from the empirical distribution of |h| over calibration entries (Eq. 4): the
    smallest observed magnitude eps with  #(|h| <= eps) >= p * N."""
    a = np.sort(np.abs(np.asarray(H, np.float64)).ravel())
    k = int(np.ceil(p * a.size))
    return float(a[k - 1]) if k >= 1 else 0.0


def threshold_indices(h: np.ndarray, eps: float) -> np.ndarray:
    """Kept channels of S_eps (Eq. 5): those with |h_i| > eps, ascending.  One token."""
    return np.flatnonzero(np.abs(np.asarray(h, np.float64)) > eps).astype(np.int32)


def silu(g: np.ndarray) -> np.ndarray:
    g = np.asarray(g, np.float64)
    return g / (1.0 + np.exp(-g))


def gqa_single_key_attention(qkv: np.ndarray, d_q: int, d_kv: int, head_dim: int) -> np.ndarray:
    """Attention core at context length 1: softmax over one key is 1, so each query
    head's output is the value head of its group.  qkv [..., d_q + 2 d_kv] -> a [..., d_q].
    (The method leaves the attention core unchanged; this exact special case stands in.)"""
    v = qkv[..., d_q + d_kv:]
    n_q, n_kv = d_q // head_dim, d_kv // head_dim
    g = n_q // n_kv
    vh = v.reshape(v.shape[:-1] + (n_kv, head_dim))
    a = np.repeat(vh, g, axis=-2)
    return a.reshape(v.shape[:-1] + (d_q,))


# --------------------------------------------------------------------------
# Decoder-layer composition (Fig. 2; Sec. 3.1 names h1..h4; Sec. 4.2-4.3)
# --------------------------------------------------------------------------


class Layer:
    """Operands of one decoder layer, already widened to fp64.
    Wqkv [d, d_q+2d_kv] and Wgu [d, 2 d_ff] are folded with Q on the input side when the
    caller rotates (h1, h3); Wo [d_q, d] and Wdown [d_ff, d] meet unrotated h2, h4 (Q = I).
    Q_attn / Q_mlp / adapter may be None.  rms_eps < 0 disables the pre-norm.
    shortcut_attn / shortcut_mlp (None = identity) are residual adapters on the two shortcuts
    (Sec. 4.2; block-level rotations use one per block, Sec. 5.4): the stream that skips a block is
    taken from the block's input basis to the basis its output projection was folded with."""

    def __init__(self, d, d_q, d_kv, d_ff, head_dim, K1, K2, K3, K4, Wqkv, Wo, Wgu, Wdown,
                 Q_attn=None, Q_mlp=None, adapter=None, rms_attn=None, rms_mlp=None,
                 rms_eps=-1.0, dtype="f16", shortcut_attn=None, shortcut_mlp=None):
        self.d, self.d_q, self.d_kv, self.d_ff, self.head_dim = d, d_q, d_kv, d_ff, head_dim
        self.K1, self.K2, self.K3, self.K4 = K1, K2, K3, K4
        self.Wqkv, self.Wo, self.Wgu, self.Wdown = Wqkv, Wo, Wgu, Wdown
        self.Q_attn, self.Q_mlp, self.adapter = Q_attn, Q_mlp, adapter
        self.rms_attn, self.rms_mlp, self.rms_eps = rms_attn, rms_mlp, rms_eps
        self.dtype = dtype
        self.shortcut_attn, self.shortcut_mlp = shortcut_attn, shortcut_mlp


def block_input(x: np.ndarray, Q, rms_scale, rms_eps: float, dtype) -> np.ndarray:
    """h1 / h3: pre-norm (optional), rotation by Q (optional), one storage rounding."""
    t = rmsnorm(x, rms_eps, rms_scale) if rms_eps >= 0 else np.asarray(x, np.float64)
    if Q is not None:
        t = rotate(t, Q)
    return round16(t, dtype)


def _select(h: np.ndarray, K: int, dtype, forced_idx=None) -> np.ndarray:
    if forced_idx is not None:
        return forced_idx
    if dtype is None:
        # unrounded run: order by |h| in fp64, ties by lower index
        order = np.argsort(-np.abs(h), kind="stable")
        return np.sort(order[:K]).astype(np.int32)
    return topk_indices(encode16(h, dtype), K)


def stage_qkv(L: Layer, h1, idx1, dtype):
    return round16(sparse_project_gather(h1, idx1, L.Wqkv), dtype)


def stage_shortcut(x, A, dtype):
    """The residual shortcut around a block: the stream itself, or x (Q_in^T Q_out) through a
    residual adapter (Sec. 4.2), one storage rounding."""
    return np.asarray(x, np.float64) if A is None else round16(rotate(x, A), dtype)


def stage_attn_out(L: Layer, x, h2, idx2, dtype):
    o = round16(sparse_project_gather(h2, idx2, L.Wo), dtype)
    return o, round16(stage_shortcut(x, L.shortcut_attn, dtype) + o, dtype)


def stage_gate_up(L: Layer, h3, idx3, dtype):
    return round16(sparse_project_gather(h3, idx3, L.Wgu), dtype)


def stage_h4(L: Layer, gu, dtype):
    return round16(silu(gu[..., :L.d_ff]) * gu[..., L.d_ff:], dtype)


def stage_down(L: Layer, x1, h4, idx4, dtype):
    dn = round16(sparse_project_gather(h4, idx4, L.Wdown), dtype)
    return dn, round16(stage_shortcut(x1, L.shortcut_mlp, dtype) + dn, dtype)


def stage_adapter(L: Layer, x2, dtype):
    return x2 if L.adapter is None else round16(rotate(x2, L.adapter), dtype)


def layer_forward(L: Layer, x: np.ndarray, rounded: bool = True, attention=None) -> dict:
    """One token through one decoder layer (Fig. 2): h1 -> q|k|v; h2 -> o; h3 -> gate|up;
    h4 = SiLU(gate)*up -> down; residual adds; optional adapter.  With rounded=True every
    tensor that crosses a kernel boundary is rounded to the layer dtype (h1, qkv, h2, o,
    x1, h3, gu, h4, down, x2, x_out); with rounded=False the whole layer is fp64.
    attention: the attention core, a function q|k|v [d_q + 2 d_kv] -> a [d_q] (the method leaves
    it unchanged, Sec. 3.1: it only sparsifies its output h2); None = the context-length-1 case.
    Returns every stage in a dict."""
    dt = L.dtype if rounded else None
    x = np.asarray(x, np.float64)
    h1 = block_input(x, L.Q_attn, L.rms_attn, L.rms_eps, dt)
    idx1 = _select(h1, L.K1, dt)
    qkv = stage_qkv(L, h1, idx1, dt)
    if attention is None:
        h2 = gqa_single_key_attention(qkv, L.d_q, L.d_kv, L.head_dim)
    else:
        h2 = round16(np.asarray(attention(qkv), np.float64), dt)
    idx2 = _select(h2, L.K2, dt)
    o, x1 = stage_attn_out(L, x, h2, idx2, dt)
    h3 = block_input(x1, L.Q_mlp, L.rms_mlp, L.rms_eps, dt)
    idx3 = _select(h3, L.K3, dt)
    gu = stage_gate_up(L, h3, idx3, dt)
    h4 = stage_h4(L, gu, dt)
    idx4 = _select(h4, L.K4, dt)
    down, x2 = stage_down(L, x1, h4, idx4, dt)
    x_out = stage_adapter(L, x2, dt)
    return dict(h1=h1, idx1=idx1, qkv=qkv, h2=h2, idx2=idx2, o=o, x1=x1, h3=h3, idx3=idx3,
                gu=gu, h4=h4, idx4=idx4, down=down, x2=x2, x_out=x_out,
                s1=stage_shortcut(x, L.shortcut_attn, dt), s2=stage_shortcut(x1, L.shortcut_mlp, dt))
