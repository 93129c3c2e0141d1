"""Pins of the oracle's 4-bit weight functions and of the magnitude-threshold sparsifier against
what round-to-nearest quantisation and Eq. 4-5 fix: error bounds, closed forms, hand-written
examples, brute force.  No GPU."""
import numpy as np
import pytest

from oracle import larosa_oracle as O


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_rtn_error_is_at_most_half_a_step_and_the_extreme_is_exact(dtype):
    rng = np.random.default_rng(5)
    W = rng.standard_normal((37, 328)) * 0.02          # 328 = 2 full groups + one of 72 columns
    codes, sb = O.quantize_rtn_w4(W, dtype)
    assert codes.shape == W.shape and sb.shape == (37, 3) and codes.min() >= 1 and codes.max() <= 15
    s = O.decode16(sb, dtype)
    deq = O.dequantize_w4(codes, sb, dtype)
    step = s[:, np.arange(328) // 128]
    assert np.all(np.abs(W - deq) <= 0.5 * step * (1 + 1e-12))
    # scale is max|w|/7 rounded once to storage; the group's extreme entry gets code 1 or 15
    for g in range(3):
        blk = W[:, g * 128:(g + 1) * 128]
        m = np.abs(blk).max(axis=1)
        assert np.array_equal(sb[:, g], O.encode16(m / 7.0, dtype))
        j = np.abs(blk).argmax(axis=1)
        q = codes[np.arange(37), g * 128 + j].astype(int) - 8
        assert np.array_equal(q, 7 * np.sign(blk[np.arange(37), j]).astype(int))


def test_rtn_brute_force_by_hand():
    # one row, one group: max 0.7 -> s = 0.1 (to f16 precision), codes follow by inspection
    W = np.array([[0.7, -0.7, 0.34, 0.36, -0.04, 0.04, 0.0, -0.149]])
    codes, sb = O.quantize_rtn_w4(W, "f16", group=8)
    s = float(O.decode16(sb, "f16")[0, 0])
    assert abs(s - 0.1) < 1e-4
    want = [int(np.rint(w / s)) + 8 for w in W[0]]       # scalar loop
    assert codes[0].tolist() == want == [15, 1, 11, 12, 8, 8, 8, 7]
    assert np.allclose(O.dequantize_w4(codes, sb, "f16", group=8)[0], (np.array(want) - 8) * s)


def test_rtn_is_idempotent_and_zero_groups_are_zero():
    rng = np.random.default_rng(6)
    W = rng.standard_normal((9, 256)) * 0.05
    W[3, :128] = 0.0
    for dtype in ("f16", "bf16"):
        codes, sb = O.quantize_rtn_w4(W, dtype)
        deq = O.dequantize_w4(codes, sb, dtype)
        assert np.all(deq[3, :128] == 0) and np.all(codes[3, :128] == 8) and sb[3, 0] == 0
        codes2, sb2 = O.quantize_rtn_w4(deq, dtype)
        keep = np.ones(256, bool)
        assert np.array_equal(sb2, sb) and np.array_equal(codes2[:, keep], codes[:, keep])


def test_pack_places_column_k_in_nibble_k():
    codes = np.array([[1, 2, 3, 4, 5, 6, 7, 8, 15, 0, 0, 0, 0, 0, 0, 9]], np.uint8)
    packed = O.pack_w4(codes)
    assert packed.dtype == np.uint32 and packed.tolist() == [[0x87654321, 0x9000000F]]
    rng = np.random.default_rng(7)
    c = rng.integers(0, 16, (5, 64)).astype(np.uint8)
    assert np.array_equal(O.unpack_w4(O.pack_w4(c)), c)


def test_w4_sparse_product_reduces_to_dense_and_to_the_masked_form():
    rng = np.random.default_rng(8)
    d, d_out = 64, 256
    W = rng.standard_normal((d, d_out)) * 0.02
    codes, sb = O.quantize_rtn_w4(W, "f16")
    deq = O.dequantize_w4(codes, sb, "f16")
    h = rng.standard_normal(d)
    full = np.arange(d, dtype=np.int32)
    assert np.allclose(O.sparse_project_w4(h, full, codes, sb, "f16"), h @ deq, rtol=0, atol=1e-14)
    idx = np.sort(rng.choice(d, 20, replace=False)).astype(np.int32)
    want = sum(h[j] * deq[j] for j in idx)               # row by row
    assert np.allclose(O.sparse_project_w4(h, idx, codes, sb, "f16"), want, rtol=0, atol=1e-14)
    assert np.allclose(O.sparse_project_w4(h, idx, codes, sb, "f16"), O.sparse_project_masked(h, idx, deq), atol=1e-14)


def test_threshold_sparsifier_definition_and_calibration():
    h = np.array([0.5, -0.2, 0.2, 0.0, -0.7, 0.21])
    assert O.threshold_indices(h, 0.2).tolist() == [0, 4, 5]          # |h| <= eps is dropped (Eq. 5)
    assert O.threshold_indices(h, 0.0).tolist() == [0, 1, 2, 4, 5]
    assert O.threshold_indices(h, 1.0).tolist() == []
    # calibrated cutoff: on the calibration data itself the dropped fraction is >= p and minimal
    rng = np.random.default_rng(9)
    H = rng.standard_normal((50, 40))
    for p in (0.25, 0.4, 0.5):
        eps = O.calibrate_threshold(H, p)
        dropped = (np.abs(H) <= eps).mean()
        assert dropped >= p
        below = np.abs(H)[np.abs(H) < eps]
        assert below.size / H.size < p                                  # any smaller cutoff drops too few
    # a Gaussian's p-quantile of |h| in closed form: eps = sqrt(2) erfinv(p)
    from scipy.special import erfinv
    G = rng.standard_normal(400000)
    assert abs(O.calibrate_threshold(G, 0.4) - np.sqrt(2) * erfinv(0.4)) < 5e-3


def test_threshold_kept_count_varies_with_token_scale_while_topk_does_not():
    """Sec. 4.1: with a fixed cutoff the kept count follows the token's scale; Top-K keeps K."""
    rng = np.random.default_rng(10)
    d, K = 512, 307
    cal = rng.standard_normal((64, d))
    eps = O.calibrate_threshold(cal, 0.4)
    counts = []
    for scale in (0.5, 1.0, 2.0):
        h = rng.standard_normal(d) * scale
        counts.append(O.threshold_indices(h, eps).size)
        bits = O.encode16(h, "f16")
        assert O.topk_indices(bits, K).size == K
    assert counts[0] < counts[1] < counts[2]
    assert abs(counts[1] / d - 0.6) < 0.08
