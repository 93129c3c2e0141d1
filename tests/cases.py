"""Test-side construction of LaRoSA layer operands from the seeded synthetic inputs.

Raw numbers come from paper_2507_01299_amd.synth; the offline method steps (PCA rotation,
folding, adapters, the one rounding to 16-bit storage) are taken with the CPU oracle, so
every operand handed to the HIP path in a parity test is an oracle-side product and never
the other way round."""
from __future__ import annotations

import dataclasses

import numpy as np

from oracle import larosa_oracle as O
from paper_2507_01299_amd import synth

RMS_EPS = 1e-5


def _store(a64: np.ndarray, dtype: str):
    """Round once to storage; return (bits uint16, exact float32 view of the stored values)."""
    bits = O.encode16(a64, dtype)
    return bits, O.decode16(bits, dtype).astype(np.float32)


@dataclasses.dataclass
class LayerCase:
    shape: synth.LayerShape
    bits: dict            # name -> uint16 arrays handed to the device (None when absent)
    layer: O.Layer        # oracle operands (stored values, widened exactly)
    dense: dict           # unfolded fp64 weights and rotations, for invariance checks
    src: synth.ActivationSource


def _dense_attention_half(X, W, shape, use_rms):
    n = O.rmsnorm(X, RMS_EPS) if use_rms else X
    v = n @ W["v"].astype(np.float64)
    qkv = np.concatenate([np.zeros((X.shape[0], shape.d_q + shape.d_kv)), v], axis=1)
    a = O.gqa_single_key_attention(qkv, shape.d_q, shape.d_kv, shape.head_dim)
    return X + a @ W["o"].astype(np.float64)


def build_block_layer(shape: synth.LayerShape, p: float, seed: int, n_cal: int,
                      use_rms: bool = True, latent: str = "gauss", with_adapter: bool = False,
                      Ks=None, with_rms_scale: bool = False, explicit_Q: bool = True) -> LayerCase:
    """One decoder layer with explicit per-block rotations Q_attn, Q_mlp (the block-level
    variant): q|k|v and gate|up are folded with Q^T on the input side; o and down see the
    unrotated h2, h4."""
    dt = shape.dtype
    src = synth.activation_source(shape.d, seed, latent=latent)
    W = synth.layer_weights(shape, seed + 100)
    Xc = src.draw(n_cal, seed + 1)
    Nc = O.rmsnorm(Xc, RMS_EPS) if use_rms else Xc
    Q_attn, _ = O.pca_rotation(O.second_moment(Nc))
    X1 = _dense_attention_half(Xc, W, shape, use_rms)
    N1 = O.rmsnorm(X1, RMS_EPS) if use_rms else X1
    Q_mlp, _ = O.pca_rotation(O.second_moment(N1))
    del Xc, Nc, X1, N1
    Wqkv = np.concatenate([W["q"], W["k"], W["v"]], axis=1).astype(np.float64)
    Wgu = np.concatenate([W["gate"], W["up"]], axis=1).astype(np.float64)
    bits, vals = {}, {}
    bits["Wqkv"], vals["Wqkv"] = _store(O.fold_input_side(Q_attn, Wqkv), dt)
    bits["Wgu"], vals["Wgu"] = _store(O.fold_input_side(Q_mlp, Wgu), dt)
    bits["Wo"], vals["Wo"] = _store(W["o"].astype(np.float64), dt)
    bits["Wdown"], vals["Wdown"] = _store(W["down"].astype(np.float64), dt)
    bits["Q_attn"], vals["Q_attn"] = _store(Q_attn, dt)
    bits["Q_mlp"], vals["Q_mlp"] = _store(Q_mlp, dt)
    A = None
    if with_adapter:
        Q_next = synth.planted_basis(shape.d, seed + 7)
        A = Q_next        # any orthogonal D x D serves as the dense mat-vec after the layer
        bits["adapter"], vals["adapter"] = _store(A, dt)
    else:
        bits["adapter"], vals["adapter"] = None, None
    if Ks is None:
        Ks = (O.kept_count(shape.d, p), O.kept_count(shape.d_q, p),
              O.kept_count(shape.d, p), O.kept_count(shape.d_ff, p))
    g_attn = g_mlp = None
    if with_rms_scale:       # learned pre-norm scales (any positive vector serves)
        rs = np.random.Generator(np.random.PCG64(seed + 9))
        bits["rms_attn"], va = _store(rs.uniform(0.5, 1.5, shape.d), dt)
        bits["rms_mlp"], vm = _store(rs.uniform(0.5, 1.5, shape.d), dt)
        g_attn, g_mlp = va.astype(np.float64), vm.astype(np.float64)
    if not explicit_Q:       # x is taken to arrive in the block's basis already: no rotation kernels
        bits["Q_attn"] = bits["Q_mlp"] = None
    layer = O.Layer(shape.d, shape.d_q, shape.d_kv, shape.d_ff, shape.head_dim, *Ks,
                    Wqkv=vals["Wqkv"], Wo=vals["Wo"], Wgu=vals["Wgu"], Wdown=vals["Wdown"],
                    Q_attn=vals["Q_attn"].astype(np.float64) if explicit_Q else None,
                    Q_mlp=vals["Q_mlp"].astype(np.float64) if explicit_Q else None,
                    adapter=None if A is None else vals["adapter"].astype(np.float64),
                    rms_attn=g_attn, rms_mlp=g_mlp,
                    rms_eps=RMS_EPS if use_rms else -1.0, dtype=dt)
    dense = dict(W=W, Q_attn=Q_attn, Q_mlp=Q_mlp, Wqkv=Wqkv, Wgu=Wgu)
    return LayerCase(shape, bits, layer, dense, src)


def tokens(case: LayerCase, B: int, seed: int):
    """B stored input tokens: (bits [B, d], fp64 values of those bits)."""
    x = case.src.draw(B, seed)
    bits = O.encode16(x, case.shape.dtype)
    return bits, O.decode16(bits, case.shape.dtype)


def build_folded_stack(shape: synth.LayerShape, n_layers: int, p: float, seed: int, n_cal: int,
                       store: bool = True):
    """n_layers decoder layers in the deployed form: the residual stream of layer l lives in
    the basis Q_l (one rotation per layer), q|k|v and gate|up carry Q_l^T on the input side,
    o and down carry Q_l on the output side, and the adapter Q_l^T Q_{l+1} follows each
    layer.  Q_l comes from PCA of the (normed) input of layer l, obtained by pushing the
    calibration tokens through the dense fp64 stack.  Returns (layers, Qs, dense weights);
    with store=False operands stay in fp64 (for invariance checks)."""
    dt = shape.dtype if store else None
    src = synth.activation_source(shape.d, seed)
    Xc = src.draw(n_cal, seed + 1)
    Ws, Qs = [], []
    X = Xc
    for l in range(n_layers):
        W = synth.layer_weights(shape, seed + 100 + 10 * l)
        Ws.append(W)
        Q, _ = O.pca_rotation(O.second_moment(O.rmsnorm(X, RMS_EPS)))
        Qs.append(Q)
        X = dense_layer_reference(W, shape, X)
    Qs.append(np.eye(shape.d))          # basis after the last layer: back to the model's own
    Ks = (O.kept_count(shape.d, p), O.kept_count(shape.d_q, p),
          O.kept_count(shape.d, p), O.kept_count(shape.d_ff, p))
    layers, bits = [], []
    for l in range(n_layers):
        W, Q = Ws[l], Qs[l]
        ops = dict(
            Wqkv=O.fold_input_side(Q, np.concatenate([W["q"], W["k"], W["v"]], axis=1)),
            Wo=O.fold_output_side(W["o"], Q),
            Wgu=O.fold_input_side(Q, np.concatenate([W["gate"], W["up"]], axis=1)),
            Wdown=O.fold_output_side(W["down"], Q),
            adapter=O.residual_adapter(Q, Qs[l + 1]))
        b = {}
        if store:
            for k in list(ops):
                b[k], v = _store(ops[k], dt)
                ops[k] = v
            ops["adapter"] = ops["adapter"].astype(np.float64)
        b["Q_attn"] = b["Q_mlp"] = None
        bits.append(b)
        layers.append(O.Layer(shape.d, shape.d_q, shape.d_kv, shape.d_ff, shape.head_dim, *Ks,
                              Wqkv=ops["Wqkv"], Wo=ops["Wo"], Wgu=ops["Wgu"], Wdown=ops["Wdown"],
                              adapter=ops["adapter"], rms_eps=RMS_EPS, dtype=shape.dtype))
    return layers, bits, Qs, Ws, src


def build_shortcut_stack(shape: synth.LayerShape, n_layers: int, p: float, seed: int, n_cal: int,
                         store: bool = True, bases=None):
    """n_layers decoder layers with block-level rotations and residual adapters on the shortcuts
    (Sec. 4.2, Sec. 5.4 "block-level"): layer l's attention block works in the basis Qa_l, its MLP
    block in Qm_l.  q|k|v carry Qa_l^T and gate|up Qm_l^T on the input side; o carries Qm_l and down
    carries Qa_{l+1} on the output side; the stream that skips the attention block goes through
    Qa_l^T Qm_l, the one that skips the MLP block through Qm_l^T Qa_{l+1}.  The stack takes the
    stream in the basis Qa_0 and returns it in the model's own basis (Qa_L = I).  Bases come from PCA
    of the (normed) block inputs reached by pushing calibration tokens through the dense fp64 stack;
    bases = (Qa list, Qm list) supplies them instead (any orthogonal matrices give a valid layer: a
    launch-shape test of a large layer need not pay for its calibration).
    Returns (layers, bits, Qa list, dense weights, source)."""
    dt = shape.dtype if store else None
    src = synth.activation_source(shape.d, seed)
    Ws = [synth.layer_weights(shape, seed + 100 + 10 * l) for l in range(n_layers)]
    if bases is not None:
        Qa, Qm = list(bases[0]), list(bases[1])
        assert len(Qa) == n_layers and len(Qm) == n_layers
    else:
        X = src.draw(n_cal, seed + 1)
        Qa, Qm = [], []
        for W in Ws:
            Qa.append(O.pca_rotation(O.second_moment(O.rmsnorm(X, RMS_EPS)))[0])
            X1 = _dense_attention_half(X, W, shape, True)
            Qm.append(O.pca_rotation(O.second_moment(O.rmsnorm(X1, RMS_EPS)))[0])
            X = dense_layer_reference(W, shape, X)
    Qa.append(None)                       # the stack returns the stream in the model's own basis (identity)
    Ks = (O.kept_count(shape.d, p), O.kept_count(shape.d_q, p),
          O.kept_count(shape.d, p), O.kept_count(shape.d_ff, p))
    layers, bits = [], []
    for l in range(n_layers):
        W = Ws[l]
        ops = dict(
            Wqkv=O.fold_input_side(Qa[l], np.concatenate([W["q"], W["k"], W["v"]], axis=1)),
            Wo=O.fold_output_side(W["o"], Qm[l]),
            Wgu=O.fold_input_side(Qm[l], np.concatenate([W["gate"], W["up"]], axis=1)),
            Wdown=O.fold_output_side(W["down"], Qa[l + 1]) if Qa[l + 1] is not None else W["down"].astype(np.float64),
            shortcut_attn=O.residual_adapter(Qa[l], Qm[l]),
            shortcut_mlp=(O.residual_adapter(Qm[l], Qa[l + 1]) if Qa[l + 1] is not None
                          else np.asarray(Qm[l], np.float64).T.copy()))
        b = {}
        if store:
            for k in list(ops):
                b[k], v = _store(ops[k], dt)
                ops[k] = v
            ops["shortcut_attn"] = ops["shortcut_attn"].astype(np.float64)
            ops["shortcut_mlp"] = ops["shortcut_mlp"].astype(np.float64)
        b["Q_attn"] = b["Q_mlp"] = b["adapter"] = None
        bits.append(b)
        layers.append(O.Layer(shape.d, shape.d_q, shape.d_kv, shape.d_ff, shape.head_dim, *Ks,
                              Wqkv=ops["Wqkv"], Wo=ops["Wo"], Wgu=ops["Wgu"], Wdown=ops["Wdown"],
                              shortcut_attn=ops["shortcut_attn"], shortcut_mlp=ops["shortcut_mlp"],
                              rms_eps=RMS_EPS, dtype=shape.dtype))
    return layers, bits, Qa, Ws, src


class CachedAttention:
    """A caller's attention core for tests: grouped-query softmax attention of one new token over a
    seeded cache of n_ctx earlier (key, value) pairs plus its own, scores q.k / sqrt(head_dim).
    Plain fp64 numpy, per head, written from the textbook definition; call it with q|k|v of one
    token ([d_q + 2 d_kv]) to get a [d_q]."""

    def __init__(self, shape: synth.LayerShape, n_ctx: int, seed: int, scale: float = 1.0):
        rng = np.random.default_rng(seed)
        self.shape = shape
        self.k_cache = rng.standard_normal((n_ctx, shape.d_kv)) * scale
        self.v_cache = rng.standard_normal((n_ctx, shape.d_kv)) * scale

    def __call__(self, qkv: np.ndarray) -> np.ndarray:
        sh = self.shape
        hd = sh.head_dim
        q, k, v = qkv[:sh.d_q], qkv[sh.d_q:sh.d_q + sh.d_kv], qkv[sh.d_q + sh.d_kv:]
        keys = np.vstack([self.k_cache, k[None, :]])
        vals = np.vstack([self.v_cache, v[None, :]])
        group = (sh.d_q // hd) // (sh.d_kv // hd)
        out = np.empty(sh.d_q)
        for head in range(sh.d_q // hd):
            kv = head // group
            qh = q[head * hd:(head + 1) * hd]
            scores = keys[:, kv * hd:(kv + 1) * hd] @ qh / np.sqrt(hd)
            w = np.exp(scores - scores.max())
            w /= w.sum()
            out[head * hd:(head + 1) * hd] = w @ vals[:, kv * hd:(kv + 1) * hd]
        return out


def dense_layer_reference(W: dict, shape: synth.LayerShape, X: np.ndarray, use_rms: bool = True,
                          attention=None) -> np.ndarray:
    """Textbook pre-norm decoder layer in fp64, no rotation, no sparsity:
    x1 = x + Attn(norm(x)) W_o, by default at context length 1 (Attn = value head of the query head's
    group), else attention(q|k|v) per token; x2 = x1 + (SiLU(n W_gate) * (n W_up)) W_down.
    Written without the oracle's layer code."""
    f = lambda a: a.astype(np.float64)
    X = np.asarray(X, np.float64)

    def norm(t):
        return t / np.sqrt((t * t).mean(axis=-1, keepdims=True) + RMS_EPS) if use_rms else t

    n = norm(X)
    v = n @ f(W["v"])
    hd = shape.head_dim
    g = (shape.d_q // hd) // (shape.d_kv // hd)
    if attention is None:
        a = np.concatenate([v[..., (i // g) * hd:(i // g + 1) * hd] for i in range(shape.d_q // hd)], axis=-1)
    else:
        qkv = np.concatenate([n @ f(W["q"]), n @ f(W["k"]), v], axis=-1)
        a = np.stack([attention(row) for row in qkv.reshape(-1, qkv.shape[-1])]).reshape(X.shape[:-1] + (shape.d_q,))
    x1 = X + a @ f(W["o"])
    n = norm(x1)
    gate = n @ f(W["gate"])
    x2 = x1 + ((gate / (1 + np.exp(-gate))) * (n @ f(W["up"]))) @ f(W["down"])
    return x2
