"""GPU parity of the single kernels, through the C ABI, against the CPU oracle on the same
seeded inputs: rotation and sparse projection within 2e-3 relative L2, Top-K indices equal."""
import numpy as np
import pytest
import torch

from oracle import larosa_oracle as O
from paper_2507_01299_amd import synth
from tests.gpu_util import REL_L2_TOL, rel_l2, stored_close, to_bits, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api(gpu_device):
    from paper_2507_01299_amd import api as A
    A.lib()
    return A


@pytest.fixture(scope="module")
def ws(api):
    return api.workspace(8, 32768, 32768, 32768)


def _heavy_vector(rng, B, d, dtype):
    v = rng.standard_normal((B, d)) * (np.arange(1, d + 1) ** -0.6)[None, :]
    v[:, rng.choice(d, 4, replace=False)] *= 20
    bits = O.encode16(v, dtype)
    return bits, O.decode16(bits, dtype)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,d", [(1, 512), (3, 1096), (1, 8), (2, 2048)])
def test_rotate_matches_oracle(api, ws, dtype, B, d):
    print(f"rotate dtype={dtype} B={B} d={d}", flush=True)
    rng = np.random.default_rng(100 + d + B)
    Q = synth.planted_basis(d, seed=d)
    qb = O.encode16(Q, dtype)
    xb, x = _heavy_vector(rng, B, d, dtype)
    h = torch.zeros(B, d, dtype=api.torch_dtype(dtype), device="cuda:0")
    api.rotate(to_dev(xb, dtype), to_dev(qb, dtype), h, dtype, ws)
    torch.cuda.synchronize()
    want = O.round16(O.rotate(x, O.decode16(qb, dtype)), dtype)      # the output is a stored 16-bit tensor
    for b in range(B):
        stored_close(to_bits(h)[b], want[b], dtype, "rotate")
    # identity rotation returns the input bits
    eye = O.encode16(np.eye(d), dtype)
    api.rotate(to_dev(xb, dtype), to_dev(eye, dtype), h, dtype, ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(h), xb)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,d,K", [(1, 512, 256), (1, 4096, 2457), (2, 4096, 1), (1, 4096, 4096), (3, 11008, 6604),
                                   (1, 14336, 8601), (2, 28672, 17203), (1, 32768, 5), (1, 8, 3), (4, 1000, 999),
                                   (1, 8192, 4915)])
def test_topk_indices_are_exact(api, dtype, B, d, K):
    print(f"topk dtype={dtype} B={B} d={d} K={K}", flush=True)
    rng = np.random.default_rng(7 * d + K)
    hb, _ = _heavy_vector(rng, B, d, dtype)
    idx = torch.full((B, K), -1, dtype=torch.int32, device="cuda:0")
    vals = torch.zeros(B, K, dtype=api.torch_dtype(dtype), device="cuda:0")
    api.topk(to_dev(hb, dtype), K, idx, dtype, vals=vals)
    torch.cuda.synchronize()
    got = idx.cpu().numpy()
    gv = to_bits(vals)
    for b in range(B):
        want = O.topk_indices(hb[b], K)
        assert np.array_equal(got[b], want)
        assert np.array_equal(gv[b], hb[b][want])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_topk_ties_and_special_values(api, dtype):
    d = 4096
    rng = np.random.default_rng(3)
    cases = []
    cases.append(np.full(d, 0x3C00, np.uint16))                                     # all equal
    few = rng.choice(np.array([0x3C00, 0xBC00, 0x3800, 0x0000, 0x8000], np.uint16), d)   # five values, many ties
    cases.append(few)
    sp = O.encode16(rng.standard_normal(d), dtype)
    inf, ninf, nan = (0x7C00, 0xFC00, 0x7E01) if dtype == "f16" else (0x7F80, 0xFF80, 0x7FC1)
    sp[[5, 900, 4095]] = [inf, nan, ninf]
    sp[[17, 18]] = [0x0000, 0x8000]
    cases.append(sp)
    cases.append(np.repeat(O.encode16(rng.standard_normal(d // 4), dtype), 4))        # GQA-style repeats
    hb = np.stack(cases)
    for K in (1, 2, 1000, 2457, 4095, 4096):
        idx = torch.full((hb.shape[0], K), -1, dtype=torch.int32, device="cuda:0")
        api.topk(to_dev(hb, dtype), K, idx, dtype)
        torch.cuda.synchronize()
        got = idx.cpu().numpy()
        for b in range(hb.shape[0]):
            assert np.array_equal(got[b], O.topk_indices(hb[b], K)), (b, K)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,d_in,d_out,K", [(1, 512, 1024, 256), (1, 512, 1000, 512), (3, 768, 1544, 300),
                                            (1, 64, 8, 1), (2, 2048, 6152, 1229), (1, 4096, 512, 4096)])
def test_sparse_gemv_matches_oracle(api, ws, dtype, B, d_in, d_out, K):
    print(f"sparse_gemv dtype={dtype} B={B} d_in={d_in} d_out={d_out} K={K}", flush=True)
    rng = np.random.default_rng(d_in + d_out + K)
    wb = O.encode16(synth.gaussian_weight(d_in, d_out, seed=d_out + K), dtype)
    hb, h = _heavy_vector(rng, B, d_in, dtype)
    idx = O.topk_batch(hb, K)
    y = torch.zeros(B, d_out, dtype=api.torch_dtype(dtype), device="cuda:0")
    dW = to_dev(wb, dtype)
    api.sparse_gemv(dW, to_dev(hb, dtype), torch.from_numpy(idx).cuda(), y, dtype, ws)
    torch.cuda.synchronize()
    W = O.decode16(wb, dtype)
    got = O.decode16(to_bits(y), dtype)
    for b in range(B):
        want = O.round16(O.sparse_project_gather(h[b], idx[b], W), dtype)   # stored 16-bit output
        stored_close(to_bits(y)[b], want, dtype, "sparse_gemv")
        assert rel_l2(got[b], O.round16(O.sparse_project_masked(h[b], idx[b], W), dtype)) <= REL_L2_TOL
    # unsorted index order is allowed and changes nothing but rounding order
    perm = np.stack([rng.permutation(idx[b]) for b in range(B)]).astype(np.int32)
    y2 = torch.zeros_like(y)
    api.sparse_gemv(dW, to_dev(hb, dtype), torch.from_numpy(perm).cuda(), y2, dtype, ws)
    torch.cuda.synchronize()
    for b in range(B):
        stored_close(to_bits(y2)[b], O.round16(O.sparse_project_gather(h[b], idx[b], W), dtype), dtype, "sparse_gemv, permuted indices")


def test_sparse_gemv_full_K_equals_dense_gemv_and_is_deterministic(api, ws):
    dtype, d_in, d_out = "f16", 1024, 2568
    rng = np.random.default_rng(5)
    wb = O.encode16(synth.gaussian_weight(d_in, d_out, seed=1), dtype)
    hb, h = _heavy_vector(rng, 2, d_in, dtype)
    ident = np.tile(np.arange(d_in, dtype=np.int32), (2, 1))
    dW, dh = to_dev(wb, dtype), to_dev(hb, dtype)
    y1 = torch.zeros(2, d_out, dtype=torch.float16, device="cuda:0")
    y2 = torch.zeros_like(y1)
    y3 = torch.zeros_like(y1)
    api.sparse_gemv(dW, dh, torch.from_numpy(ident).cuda(), y1, dtype, ws)
    api.dense_gemv(dW, dh, y2, dtype, ws)
    api.sparse_gemv(dW, dh, torch.from_numpy(ident).cuda(), y3, dtype, ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(y1), to_bits(y2))
    assert np.array_equal(to_bits(y1), to_bits(y3))
    want = O.round16(h @ O.decode16(wb, dtype), dtype)
    for b in range(2):
        stored_close(to_bits(y1)[b], want[b], dtype, "dense_gemv")


@pytest.mark.parametrize("variant,g_target,min_rows", [(0, 64, 4), (1, 2048, 1), (2, 256, 16), (0, 1024, 8),
                                                        (2, 512, 2), (1, 4096, 64)])
def test_sparse_gemv_every_launch_shape(api, variant, g_target, min_rows):
    """Each kernel shape variant and work split gives the same answer (within rounding order)."""
    dtype, d_in, d_out, K = "bf16", 1536, 3080, 777
    rng = np.random.default_rng(11)
    wb = O.encode16(synth.gaussian_weight(d_in, d_out, seed=2), dtype)
    hb, h = _heavy_vector(rng, 2, d_in, dtype)
    idx = O.topk_batch(hb, K)
    try:
        api.set_tuning(2, variant); api.set_tuning(0, g_target); api.set_tuning(1, min_rows)
        ws = api.workspace(2, d_in, d_out, K)
        y = torch.zeros(2, d_out, dtype=torch.bfloat16, device="cuda:0")
        api.sparse_gemv(to_dev(wb, dtype), to_dev(hb, dtype), torch.from_numpy(idx).cuda(), y, dtype, ws)
        torch.cuda.synchronize()
    finally:
        api.set_tuning(2, 0); api.set_tuning(0, 0); api.set_tuning(1, 8)
    W = O.decode16(wb, dtype)
    for b in range(2):
        stored_close(to_bits(y)[b], O.round16(O.sparse_project_gather(h[b], idx[b], W), dtype), dtype, "sparse_gemv")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B", [2, 4, 5, 16, 17, 33])
def test_batched_sparse_gemv_per_token_index_sets(api, dtype, B):
    """Batched variant: independent index sets per token; 2-4 tokens take the FMA kernel, 5-32 the
    matrix-core kernel, more than 32 several token groups.  Row count not a multiple of the 16-row
    tile, output width with a ragged last strip."""
    d_in, d_out, K = 1032, 1544, 413
    print(f"batched sparse_gemv dtype={dtype} B={B}", flush=True)
    rng = np.random.default_rng(1000 + B)
    wb = O.encode16(synth.gaussian_weight(d_in, d_out, seed=3), dtype)
    hb, h = _heavy_vector(rng, B, d_in, dtype)
    idx = O.topk_batch(hb, K)
    ws = api.workspace(B, d_in, d_out, K)
    y = torch.full((B, d_out), 7.0, dtype=api.torch_dtype(dtype), device="cuda:0")
    api.sparse_gemv(to_dev(wb, dtype), to_dev(hb, dtype), torch.from_numpy(idx).cuda(), y, dtype, ws)
    torch.cuda.synchronize()
    W = O.decode16(wb, dtype)
    for b in range(B):
        want = O.round16(O.sparse_project_gather(h[b], idx[b], W), dtype)
        stored_close(to_bits(y)[b], want, dtype, f"batched sparse_gemv token {b}")
    # a second call on the same workspace gives the same bits (counters were left at zero)
    y2 = torch.zeros_like(y)
    api.sparse_gemv(to_dev(wb, dtype), to_dev(hb, dtype), torch.from_numpy(idx).cuda(), y2, dtype, ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(y), to_bits(y2))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,d", [(2, 520), (8, 2048), (16, 4096), (32, 1096)])
def test_batched_rotate_matches_oracle(api, dtype, B, d):
    print(f"batched rotate dtype={dtype} B={B} d={d}", flush=True)
    rng = np.random.default_rng(200 + d + B)
    qb = O.encode16(synth.planted_basis(d, seed=d + 1), dtype)
    xb, x = _heavy_vector(rng, B, d, dtype)
    ws = api.workspace(B, d, d, d)
    h = torch.zeros(B, d, dtype=api.torch_dtype(dtype), device="cuda:0")
    api.rotate(to_dev(xb, dtype), to_dev(qb, dtype), h, dtype, ws)
    torch.cuda.synchronize()
    want = O.round16(O.rotate(x, O.decode16(qb, dtype)), dtype)
    for b in range(B):
        stored_close(to_bits(h)[b], want[b], dtype, f"batched rotate token {b}")


def test_config0_single_linear_by_its_recipe(api, ws):
    """The smallest benchmark configuration end to end through the three calls: a single linear layer
    512 x 1024, fp16, W ~ N(0, 0.02^2); tokens x = (z * s) U^T with s_i = i^-0.8 and 4 outlier channels
    x 20; Q = PCA of 2048 calibration tokens drawn the same way; W' = Q^T W rounded once.
    rotate -> Top-K (K = 256) -> column-sparse product, each stage against the oracle on the GPU's own
    stage input; and at K = d the result equals the dense product x W with the UNFOLDED weight
    (computational invariance, Sec. 3.2), to the accuracy of 16-bit storage."""
    d, d_out, K, dtype = 512, 1024, 256, "f16"
    seed = synth.seed_for(0, 0)
    src = synth.activation_source(d, seed)
    Xc = src.draw(2048, seed + 1)
    Q, lam = O.pca_rotation(O.second_moment(Xc))
    W = synth.gaussian_weight(d, d_out, seed=seed + 100).astype(np.float64)
    qb, wb = O.encode16(Q, dtype), O.encode16(O.fold_input_side(Q, W), dtype)
    xb = O.encode16(src.draw(1, seed + 5), dtype)
    x = O.decode16(xb, dtype)
    td = api.torch_dtype(dtype)
    h = torch.zeros(1, d, dtype=td, device="cuda:0")
    api.rotate(to_dev(xb, dtype), to_dev(qb, dtype), h, dtype, ws)
    torch.cuda.synchronize()
    stored_close(to_bits(h)[0], O.round16(O.rotate(x[0], O.decode16(qb, dtype)), dtype), dtype, "h = x Q")
    hb = to_bits(h)
    hv = O.decode16(hb, dtype)
    for Kc in (K, d):
        idx = torch.full((1, Kc), -1, dtype=torch.int32, device="cuda:0")
        api.topk(h, Kc, idx, dtype)
        torch.cuda.synchronize()
        want_idx = O.topk_indices(hb[0], Kc)
        assert np.array_equal(idx.cpu().numpy()[0], want_idx)
        y = torch.zeros(1, d_out, dtype=td, device="cuda:0")
        api.sparse_gemv(to_dev(wb, dtype), h, idx, y, dtype, ws)
        torch.cuda.synchronize()
        stored_close(to_bits(y)[0], O.round16(O.sparse_project_gather(hv[0], want_idx, O.decode16(wb, dtype)), dtype),
                     dtype, f"y at K = {Kc}")
        if Kc == d:
            dense = x[0] @ W        # fp64, unfolded weight, unrotated token
            got = O.decode16(to_bits(y), dtype)[0]
            # three 16-bit roundings separate the two (Q, h, W'): each is 2^-11 relative per entry
            assert rel_l2(got, dense) <= 3e-3
