"""Pins for the CPU oracle: each check ties an oracle function to something other than
itself -- a closed form, an invariant the paper states, brute force written with plain
Python loops, or a value the paper prints (tests/golden/)."""
import itertools
import math
import os
import struct

import numpy as np
import pytest
from scipy.stats import norm

from oracle import larosa_oracle as O
from paper_2507_01299_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ storage formats

def _bf16_value(u):
    return struct.unpack("<f", struct.pack("<I", int(u) << 16))[0]


def test_decode_bf16_matches_struct_unpack():
    u = np.arange(0, 65536, 7, dtype=np.uint16)
    got = O.decode16(u, "bf16")
    for ui, g in zip(u[::97], got[::97]):
        w = _bf16_value(ui)
        assert (math.isnan(w) and math.isnan(g)) or w == g


def test_decode_f16_closed_form():
    # sign, 5-bit exponent (bias 15), 10-bit mantissa
    for u in [0x0001, 0x03FF, 0x0400, 0x3C00, 0x3C01, 0x7BFF, 0xC000, 0x8001, 0x3555]:
        s = -1.0 if u & 0x8000 else 1.0
        e = (u >> 10) & 0x1F
        m = u & 0x3FF
        want = s * (m * 2.0 ** -24 if e == 0 else (1 + m / 1024.0) * 2.0 ** (e - 15))
        assert O.decode16(np.array([u], np.uint16), "f16")[0] == want


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_encode_is_round_to_nearest_even(dtype):
    # brute force: nearest representable finite value, ties to the even pattern
    pats = np.arange(0, 0x7C00 if dtype == "f16" else 0x7F80, dtype=np.uint16)   # non-negative finite
    vals = O.decode16(pats, dtype)
    rng = np.random.default_rng(5)
    x = np.concatenate([
        rng.standard_normal(4000) * 10.0 ** rng.uniform(-6, 3, 4000),
        (vals[1000:3000:7] + vals[1001:3001:7]) / 2.0,           # exact midpoints
        vals[5:4000:11],                                          # exact values
        np.array([0.0, 1e-9, 3e-8, 6e-8, 1.0, 65504.0, 1.0009765625 + 2.0 ** -12]),
    ])
    x = np.abs(x)
    x = x[x < vals[-1]]
    got = O.encode16(x, dtype)
    hi = np.searchsorted(vals, x, side="left")
    hi = np.clip(hi, 1, len(vals) - 1)
    lo = hi - 1
    dlo, dhi = x - vals[lo], vals[hi] - x
    want = np.where(dlo < dhi, lo, np.where(dhi < dlo, hi, np.where(lo % 2 == 0, lo, hi)))
    want = np.where(x == vals[hi], hi, want)
    assert np.array_equal(got.astype(np.int64), want)
    # sign symmetry
    assert np.array_equal(O.encode16(-x, dtype), got | np.uint16(0x8000))


def test_round16_identity_on_representable_values():
    for dt in ("f16", "bf16"):
        u = np.arange(0, 0x7C00 if dt == "f16" else 0x7F80, 3, dtype=np.uint16)
        assert np.array_equal(O.encode16(O.decode16(u, dt), dt), u)


# ------------------------------------------------------------------ PCA rotation

@pytest.fixture(scope="module")
def pca_case():
    d = 96
    src = synth.activation_source(d, seed=11)
    X = src.draw(1536, seed=12)
    C = O.second_moment(X)
    Q, lam = O.pca_rotation(C)
    return d, src, X, C, Q, lam


def test_second_moment_is_plain_double_loop(pca_case):
    d, src, X, C, Q, lam = pca_case
    n = X.shape[0]
    for (a, b) in [(0, 0), (3, 17), (95, 2)]:
        want = sum(X[t, a] * X[t, b] for t in range(n)) / n
        assert abs(C[a, b] - want) < 1e-12 * max(1.0, abs(want))
    assert C.shape == (d, d)


def test_Q_orthogonal_sorted_diagonalising(pca_case):
    d, src, X, C, Q, lam = pca_case
    assert np.max(np.abs(Q.T @ Q - np.eye(d))) < 1e-10
    assert np.max(np.abs(Q @ Q.T - np.eye(d))) < 1e-10
    assert np.all(np.diff(lam) <= 1e-12 * lam[0])            # descending
    D = Q.T @ C @ Q
    off = D - np.diag(np.diag(D))
    assert np.max(np.abs(off)) < 1e-8 * lam[0]
    assert np.allclose(np.diag(D), lam, rtol=0, atol=1e-9 * lam[0])
    # column i of Q is the i-th eigenvector: C q_i = lam_i q_i
    for i in (0, 1, d - 1):
        assert np.max(np.abs(C @ Q[:, i] - lam[i] * Q[:, i])) < 1e-9 * lam[0]


def test_Q_variance_concentrates_in_leading_coordinates(pca_case):
    d, src, X, C, Q, lam = pca_case
    H = O.rotate(X, Q)
    var = (H * H).mean(axis=0)
    assert np.allclose(var, lam, rtol=1e-9, atol=1e-12)
    # leading direction carries the planted outlier energy: the four x20 channels dominate it
    lead = np.abs(Q[:, 0])
    assert set(np.argsort(-lead)[:1]).issubset(set(src.outliers.tolist()))


def test_Q_recovers_planted_basis_without_outliers():
    d = 48
    src = synth.activation_source(d, seed=3, n_outliers=0, power=1.5)
    X = src.draw(200000, seed=4)
    Q, lam = O.pca_rotation(O.second_moment(X))
    M = np.abs(Q.T @ src.U)         # close to the identity on well separated leading directions
    for i in range(4):
        assert M[i, i] > 0.98


# ------------------------------------------------------------------ rotate / RMSNorm

def test_rotate_index_convention_plain_loops():
    rng = np.random.default_rng(0)
    d = 7
    x = rng.standard_normal(d)
    Q = rng.standard_normal((d, d))          # deliberately not symmetric / not orthogonal
    want = [sum(x[j] * Q[j][i] for j in range(d)) for i in range(d)]
    assert np.allclose(O.rotate(x, Q), want, rtol=1e-13, atol=1e-13)


def test_rotate_preserves_norm_and_commutes_with_rmsnorm(pca_case):
    d, src, X, C, Q, lam = pca_case
    x = X[:5]
    h = O.rotate(x, Q)
    assert np.allclose(np.linalg.norm(h, axis=1), np.linalg.norm(x, axis=1), rtol=1e-12)
    lhs = O.rmsnorm(x, 0.0)
    rhs = O.rmsnorm(O.rotate(x, Q), 0.0) @ Q.T
    assert np.max(np.abs(lhs - rhs)) < 1e-11
    eye = np.eye(d)
    assert np.array_equal(O.rotate(x, eye), x)


def test_rmsnorm_closed_form():
    x = np.array([3.0, -4.0, 0.0, 0.0])
    # mean square = 25/4
    assert np.allclose(O.rmsnorm(x, 0.0), x / 2.5)
    assert np.allclose(O.rmsnorm(x, 0.75), x / math.sqrt(7.0))
    assert np.allclose(O.rmsnorm(x, 0.0, np.array([1, 2, 3, 4.0])), x / 2.5 * np.array([1, 2, 3, 4.0]))


# ------------------------------------------------------------------ Top-K

def _brute_topk(bits, K):
    keyed = [((int(b) & 0x7FFF), i) for i, b in enumerate(bits)]
    keyed.sort(key=lambda t: (-t[0], t[1]))
    return sorted(i for _, i in keyed[:K])


def test_topk_all_permutations_and_ties_tiny():
    # every arrangement of a multiset with ties, every K
    base = [0x3C00, 0x3C00, 0xBC00, 0x4000, 0x0000, 0x8000, 0x3555]
    for perm in set(itertools.permutations(base)):
        bits = np.array(perm, np.uint16)
        for K in range(1, len(base) + 1):
            assert O.topk_indices(bits, K).tolist() == _brute_topk(perm, K)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_topk_random_vs_brute_and_invariants(dtype):
    rng = np.random.default_rng(9)
    for d, K in [(1, 1), (13, 5), (64, 64), (257, 100), (1000, 1), (4096, 2457)]:
        v = rng.standard_normal(d) * (np.arange(1, d + 1) ** -0.5)
        bits = O.encode16(v, dtype)
        idx = O.topk_indices(bits, K)
        assert idx.dtype == np.int32 and idx.shape == (K,)
        assert idx.tolist() == _brute_topk(bits.tolist(), K)
        assert np.all(np.diff(idx) > 0)                                   # distinct, ascending
        key = O.magnitude_key(bits)
        kept = np.zeros(d, bool)
        kept[idx] = True
        if K < d:
            T = key[kept].min()
            assert T >= key[~kept].max()
            ties = np.nonzero(key == T)[0]
            n_kept_ties = kept[ties].sum()
            assert np.array_equal(ties[:n_kept_ties], ties[kept[ties]])   # lowest indices among ties
        else:
            assert np.array_equal(idx, np.arange(d))


def test_topk_constructed_ties_and_special_values():
    assert O.topk_indices(np.full(10, 0x3C00, np.uint16), 4).tolist() == [0, 1, 2, 3]
    # -0 and +0 tie; Inf above finite; NaN payload above Inf
    bits = np.array([0x8000, 0x0000, 0x7C00, 0x7BFF, 0xFE00, 0xFC00, 0x0001], np.uint16)
    assert O.topk_indices(bits, 1).tolist() == [4]
    assert O.topk_indices(bits, 3).tolist() == [2, 4, 5]
    assert O.topk_indices(bits, 6).tolist() == [0, 2, 3, 4, 5, 6]
    with pytest.raises(ValueError):
        O.topk_indices(bits, 0)
    with pytest.raises(ValueError):
        O.topk_indices(bits, 8)


def test_key_is_monotone_in_magnitude():
    for dt in ("f16", "bf16"):
        u = np.arange(0, 0x7C00 if dt == "f16" else 0x7F80, dtype=np.uint16)
        v = O.decode16(u, dt)
        assert np.all(np.diff(v) > 0)
        assert np.array_equal(O.magnitude_key(u | np.uint16(0x8000)), O.magnitude_key(u))


def test_kept_fraction_is_exact_for_every_token():
    # the paper's sparsifier ablation reports zero spread of the kept fraction for Top-K
    rng = np.random.default_rng(2)
    H = O.encode16(rng.standard_normal((32, 512)) * rng.uniform(0.1, 30, (32, 1)), "f16")
    idx = O.topk_batch(H, 256)
    assert idx.shape == (32, 256)
    frac = np.array([np.count_nonzero(O.sparsify(O.decode16(H[b], "f16") + 1e-30, idx[b])) for b in range(32)]) / 512
    assert np.all(frac == 0.5) and frac.std() == 0.0


def test_kept_count_rounding():
    assert O.kept_count(4096, 0.25) == 3072
    assert O.kept_count(4096, 0.40) == 2457
    assert O.kept_count(4096, 0.50) == 2048
    assert O.kept_count(11008, 0.40) == 6604
    assert O.kept_count(14336, 0.40) == 8601
    assert O.kept_count(8192, 0.40) == 4915
    assert O.kept_count(28672, 0.40) == 17203
    assert O.kept_count(100, 0.25, alpha=1.6) == 100      # clamp to D_in
    assert O.kept_count(100, 0.999) == 1


# ------------------------------------------------------------------ sparse projection

@pytest.fixture(scope="module")
def proj_case(pca_case):
    d, src, X, C, Q, lam = pca_case
    W = synth.gaussian_weight(d, 40, seed=77).astype(np.float64)
    return W, O.fold_input_side(Q, W)


def test_fold_is_QT_times_W_plain_loops(pca_case, proj_case):
    d, src, X, C, Q, lam = pca_case
    W, Wp = proj_case
    for (i, o) in [(0, 0), (5, 39), (95, 7)]:
        want = sum(Q[j, i] * W[j, o] for j in range(d))
        assert abs(Wp[i, o] - want) < 1e-13


def test_full_K_equals_dense_product_with_unfolded_weight(pca_case, proj_case):
    d, src, X, C, Q, lam = pca_case
    W, Wp = proj_case
    x = src.draw(3, seed=90)
    for t in range(3):
        h = O.rotate(x[t], Q)
        y = O.sparse_project_gather(h, np.arange(d, dtype=np.int32), Wp)
        dense = x[t] @ W
        assert np.max(np.abs(y - dense)) < 1e-10 * np.max(np.abs(dense))


def test_gather_equals_masked_dense_and_plain_loops(pca_case, proj_case):
    d, src, X, C, Q, lam = pca_case
    W, Wp = proj_case
    x = src.draw(1, seed=91)[0]
    h = O.round16(O.rotate(x, Q), "f16")
    idx = O.topk_indices(O.encode16(h, "f16"), 37)
    a = O.sparse_project_gather(h, idx, Wp)
    b = O.sparse_project_masked(h, idx, Wp)
    assert np.max(np.abs(a - b)) < 1e-12 * np.max(np.abs(a))
    kept = set(idx.tolist())
    for o in (0, 13, 39):
        want = sum(h[i] * Wp[i, o] for i in range(d) if i in kept)
        assert abs(a[o] - want) < 1e-12
    # mask semantics: zero exactly off the kept set
    s = O.sparsify(h, idx)
    assert np.count_nonzero(s) <= 37 and np.array_equal(s[idx], h[idx])


def test_sparse_product_linearity_and_row_permutation(pca_case, proj_case):
    d, src, X, C, Q, lam = pca_case
    W, Wp = proj_case
    rng = np.random.default_rng(1)
    h1, h2 = rng.standard_normal(d), rng.standard_normal(d)
    idx = np.sort(rng.choice(d, 30, replace=False)).astype(np.int32)
    y = O.sparse_project_gather(2 * h1 - 3 * h2, idx, Wp)
    assert np.allclose(y, 2 * O.sparse_project_gather(h1, idx, Wp) - 3 * O.sparse_project_gather(h2, idx, Wp),
                       rtol=1e-12, atol=1e-14)
    perm = rng.permutation(d)
    inv = np.argsort(perm)
    # permuting channels of h and rows of W' together, and mapping the indices, changes nothing
    y2 = O.sparse_project_gather(h1[perm], np.sort(inv[idx]).astype(np.int32), Wp[perm])
    assert np.allclose(y2, O.sparse_project_gather(h1, idx, Wp), rtol=1e-12, atol=1e-14)


def test_batch_projection_uses_each_tokens_own_indices(proj_case):
    W, Wp = proj_case
    rng = np.random.default_rng(4)
    h = rng.standard_normal((3, Wp.shape[0]))
    idx = np.stack([np.sort(rng.choice(Wp.shape[0], 20, replace=False)) for _ in range(3)]).astype(np.int32)
    Y = O.sparse_project_batch(h, idx, Wp)
    for b in range(3):
        assert np.allclose(Y[b], O.sparse_project_masked(h[b], idx[b], Wp), rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ the paper's closed-form error

def _theorem_a1(k, D):
    t = norm.ppf(1.0 - k / (2.0 * D))
    return math.sqrt(1.0 - k / D - 2.0 * t * norm.pdf(t))


def test_topk_error_matches_gaussian_closed_form():
    # App. A, Theorem A.1: sqrt(E||y - y^S||^2 / E||y||^2) for iid Gaussian h and W'
    assert abs(_theorem_a1(0.75 * 4096, 4096) - 0.0914) < 5e-4
    assert abs(_theorem_a1(0.60 * 4096, 4096) - 0.1880) < 5e-4
    assert abs(_theorem_a1(0.50 * 4096, 4096) - 0.2671) < 5e-4
    rng = np.random.default_rng(17)
    D, Dout, trials = 2048, 48, 48
    for p in (0.25, 0.40, 0.50):
        K = O.kept_count(D, p)
        num = den = 0.0
        for _ in range(trials):
            h = rng.standard_normal(D)
            W = rng.standard_normal((D, Dout))
            idx = O.topk_indices(O.encode16(h, "f16"), K)
            y = h @ W
            ys = O.sparse_project_gather(h, idx, W)
            num += np.sum((y - ys) ** 2)
            den += np.sum(y ** 2)
        got = math.sqrt(num / den)
        want = _theorem_a1(K, D)
        assert abs(got - want) < 0.04 * want + 2e-3, (p, got, want)


def test_rotation_lowers_topk_error_on_structured_inputs(pca_case):
    # qualitative direction of the paper's ablation: PCA-rotated Top-K beats unrotated Top-K at equal K
    d, src, X, C, Q, lam = pca_case
    W = synth.gaussian_weight(d, 64, seed=5).astype(np.float64)
    Wp = O.fold_input_side(Q, W)
    x = src.draw(64, seed=123)
    K = 24
    e_rot = e_raw = ref = 0.0
    for t in range(64):
        y = x[t] @ W
        h = O.rotate(x[t], Q)
        yr = O.sparse_project_gather(h, O.topk_indices(O.encode16(h, "f16"), K), Wp)
        yu = O.sparse_project_gather(x[t], O.topk_indices(O.encode16(x[t], "f16"), K), W)
        e_rot += np.sum((y - yr) ** 2)
        e_raw += np.sum((y - yu) ** 2)
        ref += np.sum(y ** 2)
    assert e_rot < 0.5 * e_raw


# ------------------------------------------------------------------ alpha bookkeeping / adapter cost

def _rows(name):
    out = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                out.append(line.split())
    return out


def test_alpha_constraints_reproduce_printed_table():
    for model, a1, a2, a3, a4, M in _rows("table11_alpha.txt"):
        a1, a2, a3, a4, M = map(float, (a1, a2, a3, a4, M))
        assert abs(O.alpha_partner_attn(a1) - a2) < 1e-9, model
        assert abs(O.alpha_partner_mlp(a3, M) - a4) < 6e-3, model      # printed to 2 decimals


def test_adapter_cost_matches_printed_tflops():
    # one dense D x D mat-vec per layer per token: 2 D^2 flops, 2048 tokens per pass
    for model, L, D, orig, new in _rows("table19_adapter_tflops.txt"):
        extra = int(L) * 2 * int(D) ** 2 * 2048 / 1e12
        assert abs((float(new) - float(orig)) - extra) < 0.011, model


# ------------------------------------------------------------------ SiLU and the unrounded select

def test_silu_closed_form_values():
    """SiLU(x) = x * sigmoid(x) at points where the sigmoid is a known rational: sigmoid(ln 3) = 3/4,
    sigmoid(-ln 3) = 1/4, sigmoid(ln 2) = 2/3, sigmoid(0) = 1/2; limits x and 0 for large |x|; the
    minimum of SiLU is -0.27846454276107... at x = -1.27846454276107... (root of 1 + e^-x (1 + x) = 0)."""
    l3, l2 = math.log(3.0), math.log(2.0)
    got = O.silu(np.array([0.0, l3, -l3, l2, -l2, 1.0]))
    want = [0.0, 0.75 * l3, -0.25 * l3, (2.0 / 3.0) * l2, -(1.0 / 3.0) * l2, 1.0 / (1.0 + math.exp(-1.0))]
    assert np.allclose(got, want, rtol=0, atol=1e-15)
    assert abs(O.silu(np.array([40.0]))[0] - 40.0) < 1e-14            # x * (1 - e^-40 ...)
    assert -1e-15 < O.silu(np.array([-40.0]))[0] <= 0.0               # -40 e^-40
    x0 = -1.2784645427610737
    assert abs(O.silu(np.array([x0]))[0] - x0 / (1.0 + math.exp(-x0))) < 1e-15
    assert abs(O.silu(np.array([x0]))[0] + 0.27846454276107380) < 1e-12
    xs = np.linspace(-6, 6, 2001)
    assert np.all(O.silu(xs) >= O.silu(np.array([x0]))[0] - 1e-15)    # it is the minimum
    # odd-part identity: SiLU(x) - SiLU(-x) = x
    assert np.allclose(O.silu(xs) - O.silu(-xs), xs, rtol=0, atol=1e-14)


def test_unrounded_select_matches_brute_force_sort_below_full_K():
    """The fp64 (unrounded) layer run orders by |h| in fp64 with the lower index first among equals:
    against a plain Python sort, K < d, with exact ties planted."""
    rng = np.random.default_rng(17)
    for d, K in ((12, 5), (64, 1), (257, 100), (1000, 999)):
        h = rng.standard_normal(d)
        h[rng.choice(d, d // 4, replace=False)] = rng.choice([0.5, -0.5, 2.0])      # ties, both signs
        got = O._select(h, K, None)
        brute = sorted(sorted(range(d), key=lambda i: (-abs(h[i]), i))[:K])
        assert got.tolist() == brute
        assert got.dtype == np.int32 and np.all(np.diff(got) > 0)
    # and a layer run: every index set of the unrounded run is the brute-force set of its own stage input
    shape = synth.LayerShape("pin", 64, 64, 32, 96, 16, "f16")
    from tests import cases
    case = cases.build_block_layer(shape, 0.5, seed=5, n_cal=256)
    x = case.src.draw(1, seed=9)[0]
    r = O.layer_forward(case.layer, x, rounded=False)
    for hn, inn, K in (("h1", "idx1", case.layer.K1), ("h2", "idx2", case.layer.K2), ("h3", "idx3", case.layer.K3),
                       ("h4", "idx4", case.layer.K4)):
        h = r[hn]
        assert K < h.size
        assert r[inn].tolist() == sorted(sorted(range(h.size), key=lambda i: (-abs(h[i]), i))[:K])
