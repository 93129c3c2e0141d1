"""Pins for the oracle's decoder-layer composition: computational invariance against a
textbook dense layer written independently (tests/cases.dense_layer_reference)."""
import numpy as np

from oracle import larosa_oracle as O
from paper_2507_01299_amd import synth
from tests import cases

SMALL = synth.LayerShape("small", 64, 64, 32, 176, 16, "f16")


def _full_K(layer):
    layer.K1, layer.K2, layer.K3, layer.K4 = layer.d, layer.d_q, layer.d, layer.d_ff


def test_block_layer_full_K_equals_dense_layer():
    case = cases.build_block_layer(SMALL, 0.4, seed=21, n_cal=512)
    L = case.layer
    # unrounded operands: fold in fp64 without the storage rounding
    L.Wqkv = O.fold_input_side(case.dense["Q_attn"], case.dense["Wqkv"])
    L.Wgu = O.fold_input_side(case.dense["Q_mlp"], case.dense["Wgu"])
    L.Wo = case.dense["W"]["o"].astype(np.float64)
    L.Wdown = case.dense["W"]["down"].astype(np.float64)
    L.Q_attn, L.Q_mlp = case.dense["Q_attn"], case.dense["Q_mlp"]
    _full_K(L)
    X = case.src.draw(4, seed=5)
    want = cases.dense_layer_reference(case.dense["W"], SMALL, X)
    for t in range(4):
        got = O.layer_forward(L, X[t], rounded=False)["x_out"]
        assert np.max(np.abs(got - want[t])) < 1e-9 * np.max(np.abs(want[t]))


def test_folded_stack_with_adapters_full_K_equals_dense_stack():
    n_layers = 3
    layers, _, Qs, Ws, src = cases.build_folded_stack(SMALL, n_layers, 0.4, seed=31, n_cal=512, store=False)
    for A in (l.adapter for l in layers):
        assert np.max(np.abs(A.T @ A - np.eye(SMALL.d))) < 1e-10        # adapters are orthogonal
    X = src.draw(3, seed=9)
    want = X
    for W in Ws:
        want = cases.dense_layer_reference(W, SMALL, want)
    for t in range(3):
        xt = O.rotate(X[t], Qs[0])                   # Q_0 folded into the embedding
        for L in layers:
            _full_K(L)
            xt = O.layer_forward(L, xt, rounded=False)["x_out"]
        assert np.max(np.abs(xt - want[t])) < 1e-9 * np.max(np.abs(want[t]))


def test_shortcut_adapter_stack_full_K_equals_dense_stack():
    """Block-level rotations with a residual adapter on each shortcut (Sec. 4.2, Sec. 5.4): at full K
    the stack, entered in the first block's basis, returns the dense stack's output."""
    n_layers = 2
    layers, _, Qa, Ws, src = cases.build_shortcut_stack(SMALL, n_layers, 0.4, seed=51, n_cal=512, store=False)
    for L in layers:
        for A in (L.shortcut_attn, L.shortcut_mlp):
            assert np.max(np.abs(A.T @ A - np.eye(SMALL.d))) < 1e-10
        assert L.Q_attn is None and L.Q_mlp is None and L.adapter is None      # every rotation is absorbed
    X = src.draw(3, seed=9)
    want = X
    for W in Ws:
        want = cases.dense_layer_reference(W, SMALL, want)
    for t in range(3):
        xt = O.rotate(X[t], Qa[0])
        for L in layers:
            _full_K(L)
            r = O.layer_forward(L, xt, rounded=False)
            # the shortcut values are the adapters applied to the block inputs
            assert np.allclose(r["s1"], xt @ L.shortcut_attn, atol=1e-12)
            assert np.allclose(r["s2"], r["x1"] @ L.shortcut_mlp, atol=1e-12)
            xt = r["x_out"]
        assert np.max(np.abs(xt - want[t])) < 1e-9 * np.max(np.abs(want[t]))
    # and it is the same function as the stack with one adapter after each layer when both use the
    # same per-layer basis: adapter on the shortcut + output-side fold == adapter after the add
    rng = np.random.default_rng(3)
    d = SMALL.d
    Ql, Qn = synth.planted_basis(d, 71), synth.planted_basis(d, 72)
    x1, y = rng.standard_normal(d), rng.standard_normal(d)             # y: block output in basis Ql
    A = O.residual_adapter(Ql, Qn)
    assert np.allclose((x1 + y) @ A, x1 @ A + y @ A, atol=1e-12)


def test_sparse_layer_is_close_to_dense_and_keeps_exact_counts():
    case = cases.build_block_layer(SMALL, 0.25, seed=41, n_cal=512)
    L = case.layer
    xb, x = cases.tokens(case, 2, seed=6)
    for t in range(2):
        r = O.layer_forward(L, x[t], rounded=True)
        for name, K, n in (("idx1", L.K1, L.d), ("idx2", L.K2, L.d_q), ("idx3", L.K3, L.d), ("idx4", L.K4, L.d_ff)):
            idx = r[name]
            assert idx.shape == (K,) and np.all(np.diff(idx) > 0) and idx[0] >= 0 and idx[-1] < n
        # stored tensors are representable in the layer dtype
        for name in ("h1", "qkv", "o", "x1", "h3", "gu", "h4", "down", "x2", "x_out"):
            assert np.array_equal(O.round16(r[name], "f16"), r[name])
        # stage functions replayed on the run's own tensors give the same stages (teacher forcing)
        assert np.array_equal(O.stage_qkv(L, r["h1"], r["idx1"], "f16"), r["qkv"])
        assert np.array_equal(O.stage_h4(L, r["gu"], "f16"), r["h4"])
        assert np.array_equal(O.stage_down(L, r["x1"], r["h4"], r["idx4"], "f16")[1], r["x2"])
        dense = cases.dense_layer_reference(case.dense["W"], SMALL, x[t])
        rel = np.linalg.norm(r["x_out"] - dense) / np.linalg.norm(dense)
        assert rel < 0.2


def test_attention_core_hook_default_and_full_K_dense():
    """The attention core is the caller's (Sec. 3.1: the method only sparsifies its output h2).  Passing
    the context-length-1 case explicitly changes nothing; with a softmax attention over a cache, the
    folded layer at full K, un-rotated, is the textbook dense layer with that attention; and at 40 %
    sparsity h2 is the attention's rounded output and the later stages are the staged functions of it."""
    layers, _, Qa, Ws, src = cases.build_shortcut_stack(SMALL, 1, 0.4, seed=77, n_cal=512, store=False)
    L = layers[0]
    att = cases.CachedAttention(SMALL, n_ctx=5, seed=3)
    X = src.draw(2, seed=11)
    for t in range(2):
        xt = O.rotate(X[t], Qa[0])
        a = O.layer_forward(L, xt, rounded=True)
        b = O.layer_forward(L, xt, rounded=True,
                            attention=lambda qkv: O.gqa_single_key_attention(qkv, L.d_q, L.d_kv, L.head_dim))
        for k in a:
            assert np.array_equal(a[k], b[k]), k
        r = O.layer_forward(L, xt, rounded=True, attention=att)
        assert np.array_equal(r["h2"], O.round16(att(r["qkv"]), L.dtype))
        assert not np.allclose(r["h2"], a["h2"])                      # the cache does change the output
        assert np.array_equal(r["idx2"], O.topk_indices(O.encode16(r["h2"], L.dtype), L.K2))
        o, x1 = O.stage_attn_out(L, xt, r["h2"], r["idx2"], L.dtype)
        assert np.array_equal(r["o"], o) and np.array_equal(r["x1"], x1)
    _full_K(L)
    want = cases.dense_layer_reference(Ws[0], SMALL, X, attention=att)
    for t in range(2):
        got = O.layer_forward(L, O.rotate(X[t], Qa[0]), rounded=False, attention=att)["x_out"]
        assert np.max(np.abs(got - want[t])) < 1e-9 * np.max(np.abs(want[t]))
    # the attention reference itself: with q = 0 every score is equal, so the output is the mean of the values
    one = cases.CachedAttention(SMALL, n_ctx=1, seed=4)
    qkv = np.zeros(SMALL.d_q + 2 * SMALL.d_kv)
    np.testing.assert_allclose(one(qkv)[:SMALL.head_dim], 0.5 * one.v_cache[0, :SMALL.head_dim])
