"""GPU parity of the decoder layer (larosa_layer_forward) against the CPU oracle, stage by
stage through the trace, on seeded synthetic layers of the paper's model shapes."""
import numpy as np
import pytest
import torch

from oracle import larosa_oracle as O
from paper_2507_01299_amd import synth
from tests import cases
from tests.gpu_util import check_layer_trace, device_layer, free_run_index_disagreement, to_bits, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api(gpu_device):
    from paper_2507_01299_amd import api as A
    A.lib()
    return A


def _run_layer(api, case, B, seed, trace=True):
    dt = case.shape.dtype
    xb, _ = cases.tokens(case, B, seed)
    dl = device_layer(case)
    ws = api.Workspace(dl.workspace_bytes(B))
    x = to_dev(xb, dt)
    out = torch.zeros_like(x)
    tr = dl.trace_buffers(B) if trace else None
    api.layer_forward(dl, x, out, ws, tr)
    torch.cuda.synchronize()
    return xb, out, tr, dl, ws


@pytest.fixture(params=[(1, 1), (1, 0), (0, 1)], ids=["fused", "fused-no-histograms", "separate"])
def fused_mode(api, request):
    """Run the layer with the Top-K fused into the projection kernels -- with the down projection taking its
    threshold from the histograms the gate|up launch builds, and with every launch selecting for itself --
    and with the Top-K as separate kernels."""
    api.set_tuning(3, request.param[0])
    api.set_tuning(9, request.param[1])
    yield request.param
    api.set_tuning(3, 1)
    api.set_tuning(9, 1)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("adapter", [False, True])
def test_tiny_layer_every_stage(api, fused_mode, dtype, adapter):
    print(f"tiny layer dtype={dtype} adapter={adapter} fused={fused_mode}", flush=True)
    shape = synth.LayerShape("tiny", 256, 256, 128, 704, 32, dtype)
    case = cases.build_block_layer(shape, 0.4, seed=51, n_cal=1024, with_adapter=adapter)
    xb, out, tr, dl, ws = _run_layer(api, case, 3, seed=8)
    worst = check_layer_trace(case.layer, xb, tr, out)
    print("worst rel-L2 per stage:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
    # a run without trace buffers gives the same output bits
    out2 = torch.zeros_like(out)
    api.layer_forward(dl, to_dev(xb, dtype), out2, ws, None)
    torch.cuda.synchronize()
    assert np.array_equal(to_bits(out), to_bits(out2))


@pytest.mark.parametrize("B", [1, 2])
@pytest.mark.parametrize("Ks", [(256, 256, 256, 704), (1, 1, 1, 1), (255, 1, 256, 703)])
def test_degenerate_kept_counts(api, fused_mode, B, Ks):
    """Everything kept (K = width: the sparsifier is the identity), one value kept, and one short of everything: the
    select's thresholds sit at the ends of the key range, and the handed-down histograms are read at their first and
    last bins."""
    print(f"degenerate kept counts B={B} K={Ks} fused={fused_mode}", flush=True)
    shape = synth.LayerShape("tiny", 256, 256, 128, 704, 32, "bf16")
    case = cases.build_block_layer(shape, 0.4, seed=77, n_cal=1024, Ks=Ks)
    xb, out, tr, dl, ws = _run_layer(api, case, B, seed=3)
    check_layer_trace(case.layer, xb, tr, out)


@pytest.mark.parametrize("B", [17, 40, 70])
def test_large_batches_span_several_token_groups(api, B):
    """The batched kernels handle 16 or 32 tokens per group: batches that fill one group partly,
    two groups, and three groups with a ragged last one; both layer forms."""
    shape = synth.LayerShape("tiny", 256, 256, 128, 704, 32, "bf16")
    case = cases.build_block_layer(shape, 0.4, seed=91, n_cal=1024, with_adapter=True)
    xb, out, tr, dl, ws = _run_layer(api, case, B, seed=12)
    check_layer_trace(case.layer, xb, tr, out)
    layers, bits, Qa, _, src = cases.build_shortcut_stack(shape, 1, 0.4, seed=93, n_cal=1024)
    sc = cases.LayerCase(shape, bits[0], layers[0], {}, src)
    xb = O.encode16(O.rotate(src.draw(B, seed=13), Qa[0]), "bf16")
    dl = device_layer(sc)
    ws = api.Workspace(dl.workspace_bytes(B))
    x = to_dev(xb, "bf16")
    out = torch.zeros_like(x)
    tr = dl.trace_buffers(B)
    api.layer_forward(dl, x, out, ws, tr)
    torch.cuda.synchronize()
    check_layer_trace(layers[0], xb, tr, out)


@pytest.mark.parametrize("seed", list(range(12)))
def test_seeded_random_shapes_and_kept_counts(api, seed):
    """Seeded random layer shapes (every width a multiple of 8, GQA groups of 1-4), random kept counts
    including the extremes, batch 1-5, both dtypes, explicit and shortcut forms."""
    rng = np.random.default_rng(7000 + seed)
    head_dim = int(rng.choice([8, 16, 24, 32]))
    kv_heads = int(rng.integers(1, 5))
    group = int(rng.integers(1, 5))
    d_kv, d_q = head_dim * kv_heads, head_dim * kv_heads * group
    d = 8 * int(rng.integers(4, 90))
    d_ff = 8 * int(rng.integers(4, 200))
    dtype = "f16" if seed % 2 == 0 else "bf16"
    shape = synth.LayerShape(f"rand{seed}", d, d_q, d_kv, d_ff, head_dim, dtype)

    def pick(n):
        return int(rng.choice([1, n, max(1, n // 2), int(rng.integers(1, n + 1))]))

    Ks = (pick(d), pick(d_q), pick(d), pick(d_ff))
    B = int(rng.integers(1, 6))
    print(f"shape d={d} d_q={d_q} d_kv={d_kv} d_ff={d_ff} head_dim={head_dim} {dtype} Ks={Ks} B={B}", flush=True)
    case = cases.build_block_layer(shape, 0.4, seed=100 + seed, n_cal=max(256, 2 * d), Ks=Ks,
                                   with_adapter=bool(seed % 3 == 0))
    xb, out, tr, dl, ws = _run_layer(api, case, B, seed=seed)
    check_layer_trace(case.layer, xb, tr, out)
    layers, bits, Qa, _, src = cases.build_shortcut_stack(shape, 1, 0.4, seed=200 + seed, n_cal=max(256, 2 * d))
    L = layers[0]
    L.K1, L.K2, L.K3, L.K4 = Ks
    sc = cases.LayerCase(shape, bits[0], L, {}, src)
    xb = O.encode16(O.rotate(src.draw(B, seed=seed), Qa[0]), dtype)
    dl = device_layer(sc)
    ws = api.Workspace(dl.workspace_bytes(B))
    x = to_dev(xb, dtype)
    out = torch.zeros_like(x)
    tr = dl.trace_buffers(B)
    api.layer_forward(dl, x, out, ws, tr)
    torch.cuda.synchronize()
    check_layer_trace(L, xb, tr, out)


def test_ragged_layer_shapes(api, fused_mode):
    """Widths that are not multiples of the 512-column strip or of the per-lane element run, GQA
    with 4 query heads per value head, K values at both extremes."""
    shape = synth.LayerShape("ragged", 328, 384, 96, 1000, 24, "bf16")
    for Ks in ((1, 384, 327, 999), (328, 1, 1, 1), (200, 100, 150, 613)):
        case = cases.build_block_layer(shape, 0.4, seed=71, n_cal=768, Ks=Ks)
        xb, out, tr, dl, ws = _run_layer(api, case, 2, seed=4)
        check_layer_trace(case.layer, xb, tr, out)


@pytest.mark.parametrize("B", [1, 3, 6])
@pytest.mark.parametrize("explicit_Q", [True, False])
def test_learned_prenorm_scales_and_no_norm(api, fused_mode, B, explicit_Q):
    """Pre-norm with a learned per-channel scale (applied in fp32 in front of the rotation, or inside
    the fused prologue when there is no explicit rotation), and a layer with the pre-norm disabled."""
    shape = synth.LayerShape("tiny", 256, 256, 64, 704, 32, "f16")
    for use_rms, scale in ((True, True), (False, False)):
        case = cases.build_block_layer(shape, 0.4, seed=81, n_cal=768, use_rms=use_rms, with_rms_scale=scale,
                                       explicit_Q=explicit_Q, with_adapter=True)
        xb, out, tr, dl, ws = _run_layer(api, case, B, seed=5)
        check_layer_trace(case.layer, xb, tr, out)


def test_folded_stack_tiny(api, fused_mode):
    """Deployed form: no explicit rotations, per-layer adapters, x carried in the layer basis."""
    shape = synth.LayerShape("tiny", 256, 256, 128, 704, 32, "f16")
    layers, bits, Qs, Ws, src = cases.build_folded_stack(shape, 4, 0.4, seed=61, n_cal=1024)
    x0 = O.rotate(src.draw(2, seed=9), Qs[0])
    xb = O.encode16(x0, "f16")
    cur = to_dev(xb, "f16")
    for L, b in zip(layers, bits):
        case = cases.LayerCase(shape, b, L, {}, src)
        dl = device_layer(case)
        ws = api.Workspace(dl.workspace_bytes(2))
        out = torch.zeros_like(cur)
        tr = dl.trace_buffers(2)
        api.layer_forward(dl, cur, out, ws, tr)
        torch.cuda.synchronize()
        check_layer_trace(L, to_bits(cur), tr, out)
        cur = out


@pytest.mark.parametrize("B", [1, 3])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_shortcut_adapter_stack_tiny(api, fused_mode, B, dtype):
    """Block-level rotations with every rotation absorbed and a residual adapter on each shortcut; at
    batch 1 with the fused kernels each adapter shares the launch of the block's first projection."""
    shape = synth.LayerShape("tiny", 256, 256, 128, 704, 32, dtype)
    layers, bits, Qa, Ws, src = cases.build_shortcut_stack(shape, 3, 0.4, seed=63, n_cal=1024)
    xb = O.encode16(O.rotate(src.draw(B, seed=9), Qa[0]), dtype)
    cur = to_dev(xb, dtype)
    for L, b in zip(layers, bits):
        case = cases.LayerCase(shape, b, L, {}, src)
        dl = device_layer(case)
        ws = api.Workspace(dl.workspace_bytes(B))
        out = torch.zeros_like(cur)
        tr = dl.trace_buffers(B)
        assert "s1" in tr and "s2" in tr
        api.layer_forward(dl, cur, out, ws, tr)
        torch.cuda.synchronize()
        check_layer_trace(L, to_bits(cur), tr, out)
        # without trace buffers the result is the same bits
        out2 = torch.zeros_like(cur)
        api.layer_forward(dl, cur, out2, ws)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
        cur = out


@pytest.mark.parametrize("B", [1, 3])
@pytest.mark.parametrize("form", ["shortcut", "explicit"])
def test_layer_split_around_a_callers_attention_core(api, fused_mode, B, form):
    """larosa_layer_qkv, then softmax attention over a cache computed by the caller (here: fp64 numpy on
    the GPU's own q|k|v), then larosa_layer_after_attention: every stage equals the oracle's, with h2
    exactly the caller's vector."""
    shape = synth.LayerShape("gqa", 1096, 1024, 256, 1160, 64, "bf16")
    if form == "shortcut":
        layers, bits, Qa, _, src = cases.build_shortcut_stack(shape, 1, 0.4, seed=81, n_cal=2048)
        case = cases.LayerCase(shape, bits[0], layers[0], {}, src)
        xb = O.encode16(O.rotate(src.draw(B, seed=21), Qa[0]), shape.dtype)
    else:
        case = cases.build_block_layer(shape, 0.4, seed=82, n_cal=2048)
        xb, _ = cases.tokens(case, B, 22)
    L = case.layer
    print(f"split layer form={form} B={B} mode={fused_mode}", flush=True)
    dl = device_layer(case)
    ws = api.Workspace(dl.workspace_bytes(B))
    x = to_dev(xb, shape.dtype)
    tr = dl.trace_buffers(B)
    api.layer_qkv(dl, x, tr["qkv"], tr.get("s1"), ws, tr)
    torch.cuda.synchronize()
    att = cases.CachedAttention(shape, n_ctx=7, seed=5, scale=0.05)
    qkv = O.decode16(to_bits(tr["qkv"]), shape.dtype)
    attn_bits = O.encode16(np.stack([att(qkv[b]) for b in range(B)]), shape.dtype)
    out = torch.zeros_like(x)
    residual = tr["s1"] if L.shortcut_attn is not None else x
    api.layer_after_attention(dl, residual, to_dev(attn_bits, shape.dtype), out, ws, tr)
    torch.cuda.synchronize()
    worst = check_layer_trace(L, xb, tr, out, attn_bits=attn_bits)
    assert not np.array_equal(attn_bits, O.encode16(O.gqa_single_key_attention(qkv, L.d_q, L.d_kv, L.head_dim),
                                                    shape.dtype))      # not the built-in stand-in
    print("worst rel-L2 per stage:", {k: f"{v:.1e}" for k, v in worst.items()}, flush=True)


@pytest.mark.parametrize("side_g,main_g", [(256, 256), (64, 448), (512, 512), (8, 16)])
def test_shortcut_adapter_launch_shapes(api, side_g, main_g):
    """Every split of the shared launch between the projection and its adapter gives the same stages."""
    shape = synth.LayerShape("ragged", 1096, 1096, 1096, 1160, 8, "f16")
    layers, bits, Qa, Ws, src = cases.build_shortcut_stack(shape, 1, 0.4, seed=65, n_cal=2048)
    api.set_tuning(5, main_g)
    api.set_tuning(6, side_g)
    try:
        case = cases.LayerCase(shape, bits[0], layers[0], {}, src)
        xb = O.encode16(O.rotate(src.draw(1, seed=3), Qa[0]), "f16")
        dl = device_layer(case)
        ws = api.Workspace(dl.workspace_bytes(1))
        x = to_dev(xb, "f16")
        out = torch.zeros_like(x)
        tr = dl.trace_buffers(1)
        api.layer_forward(dl, x, out, ws, tr)
        torch.cuda.synchronize()
        check_layer_trace(layers[0], xb, tr, out)
    finally:
        api.set_tuning(5, 0)
        api.set_tuning(6, 0)


@pytest.mark.parametrize("B,form", [(1, "shortcut"), (1, "explicit"), (4, "explicit"), (3, "shortcut")])
def test_layer_in_a_hip_graph_replays_to_the_eager_bits(api, B, form):
    """The bench times graph replays: a captured layer step must give the eager result on every replay,
    with other work and synchronisations between the replays (arrival counters return to zero by
    themselves, nothing in the step is a memset)."""
    shape = synth.LayerShape("tiny", 256, 256, 128, 704, 32, "f16")
    if form == "shortcut":
        layers, bits, Qa, _, src = cases.build_shortcut_stack(shape, 1, 0.4, seed=67, n_cal=1024)
        case = cases.LayerCase(shape, bits[0], layers[0], {}, src)
    else:
        case = cases.build_block_layer(shape, 0.4, seed=67, n_cal=1024, with_adapter=True)
    xb, _ = cases.tokens(case, B, seed=4)
    dl = device_layer(case)
    ws = api.Workspace(dl.workspace_bytes(B))
    x = to_dev(xb, "f16")
    eager = torch.zeros_like(x)
    api.layer_forward(dl, x, eager, ws)
    torch.cuda.synchronize()
    out = torch.zeros_like(x)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        api.layer_forward(dl, x, out, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        api.layer_forward(dl, x, out, ws)
    for rep in range(4):
        out.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
        other = torch.zeros_like(x)
        api.layer_forward(dl, x, other, ws)          # eager work on the same workspace between replays
        torch.cuda.synchronize()
        assert torch.equal(other.view(torch.int16), eager.view(torch.int16))


@pytest.mark.parametrize("B", [1, 3, 17])
@pytest.mark.parametrize("form", ["shortcut", "explicit"])
def test_untraced_run_gives_the_traced_output(api, B, form):
    """A run without trace buffers (what the bench times) skips the stores of the intermediate tensors and, in the
    batched path, of the index lists; the layer output must keep its bits, and the traced run is the one the
    oracle checks stage by stage."""
    shape = synth.LayerShape("tiny", 256, 256, 128, 704, 32, "bf16")
    if form == "shortcut":
        layers, bits, Qa, _, src = cases.build_shortcut_stack(shape, 1, 0.4, seed=91, n_cal=1024)
        case = cases.LayerCase(shape, bits[0], layers[0], {}, src)
    else:
        case = cases.build_block_layer(shape, 0.4, seed=91, n_cal=1024, with_adapter=True)
    print(f"untraced vs traced B={B} form={form}", flush=True)
    xb, traced, tr, dl, ws = _run_layer(api, case, B, seed=6)
    check_layer_trace(case.layer, xb, tr, traced)
    plain = torch.zeros_like(traced)
    api.layer_forward(dl, to_dev(xb, "bf16"), plain, ws)
    torch.cuda.synchronize()
    assert torch.equal(plain.view(torch.int16), traced.view(torch.int16))


def test_config1_llama2_7b_shortcut_form_full_size(api):
    """The benchmark layer in the deployed block-level form: rotations absorbed, two 4096 x 4096
    residual adapters on the shortcuts, 40 % sparsity, batch 1."""
    print("building llama2-7b shortcut-form case", flush=True)
    shape = synth.SHAPES["llama2-7b"]
    layers, bits, Qa, Ws, src = cases.build_shortcut_stack(shape, 1, 0.4, seed=synth.seed_for(1, 0), n_cal=4096)
    L = layers[0]
    assert (L.K1, L.K2, L.K3, L.K4) == (2457, 2457, 2457, 6604)
    case = cases.LayerCase(shape, bits[0], L, {}, src)
    xb = O.encode16(O.rotate(src.draw(1, synth.seed_for(1, 5)), Qa[0]), "f16")
    dl = device_layer(case)
    ws = api.Workspace(dl.workspace_bytes(1))
    x = to_dev(xb, "f16")
    out = torch.zeros_like(x)
    tr = dl.trace_buffers(1)
    print("running", flush=True)
    api.layer_forward(dl, x, out, ws, tr)
    torch.cuda.synchronize()
    worst = check_layer_trace(L, xb, tr, out)
    print("worst rel-L2 per stage:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
    # the same layer at the kept counts of the paper's own allocation for this model (App. B table of optimal
    # coefficients: alpha = 0.90 / 1.30 / 0.80 / 1.15 at 40 %; counts from tests/golden/appendix_b_kept_counts.txt)
    Ks = _golden_counts("LLaMA2-7B", "0.40")
    assert Ks == (2211, 3194, 1966, 7587)
    L.K1, L.K2, L.K3, L.K4 = Ks
    dl.c.K1, dl.c.K2, dl.c.K3, dl.c.K4 = Ks
    ws = api.Workspace(dl.workspace_bytes(1))
    tr = dl.trace_buffers(1)
    print("running at the App. B counts", Ks, flush=True)
    api.layer_forward(dl, x, out, ws, tr)
    torch.cuda.synchronize()
    assert tuple(tr[k].shape[1] for k in ("idx1", "idx2", "idx3", "idx4")) == Ks
    worst = check_layer_trace(L, xb, tr, out)
    print("worst rel-L2 per stage:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)


def _golden_counts(model, p):
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "appendix_b_kept_counts.txt")) as f:
        for line in f:
            t = line.split()
            if t and t[0] == model and t[1] == p:
                return tuple(int(v) for v in t[4:8])
    raise KeyError((model, p))


def test_config1_llama2_7b_layer_full_size(api):
    """The benchmark configuration: LLaMA2-7B-shaped layer, fp16, 40 % sparsity, batch 1, with
    PCA rotations from 4096 synthetic calibration tokens."""
    print("building llama2-7b case", flush=True)
    case = cases.build_block_layer(synth.SHAPES["llama2-7b"], 0.4, seed=synth.seed_for(1, 0), n_cal=4096)
    assert (case.layer.K1, case.layer.K2, case.layer.K3, case.layer.K4) == (2457, 2457, 2457, 6604)
    print("running", flush=True)
    xb, out, tr, dl, ws = _run_layer(api, case, 1, seed=synth.seed_for(1, 5))
    worst = check_layer_trace(case.layer, xb, tr, out)
    print("worst rel-L2 per stage:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
    print("free-run index disagreements:", free_run_index_disagreement(case.layer, xb, tr), flush=True)


def test_config2_llama3_8b_gqa_bf16_batched_sparsities(api):
    """LLaMA3-8B-shaped layer (GQA, d_kv = 1024), bf16: every cell of decode batch 1 / 4 / 16 (independent
    per-token index sets) x sparsity 25 / 40 / 50 %, each stage of each token against the oracle."""
    shape = synth.SHAPES["llama3-8b"]
    print("building llama3-8b case", flush=True)
    case = cases.build_block_layer(shape, 0.4, seed=synth.seed_for(2, 0), n_cal=4096)
    L = case.layer
    dl = device_layer(case)
    for p, B in [(p, B) for p in (0.25, 0.40, 0.50) for B in (1, 4, 16)]:
        Ks = (O.kept_count(shape.d, p), O.kept_count(shape.d_q, p), O.kept_count(shape.d, p),
              O.kept_count(shape.d_ff, p))
        assert Ks in ((3072, 3072, 3072, 10752), (2457, 2457, 2457, 8601), (2048, 2048, 2048, 7168))
        L.K1, L.K2, L.K3, L.K4 = Ks
        dl.c.K1, dl.c.K2, dl.c.K3, dl.c.K4 = Ks
        print(f"sparsity {p} batch {B}", flush=True)
        xb, _ = cases.tokens(case, B, synth.seed_for(2, 5) + B)
        ws = api.Workspace(dl.workspace_bytes(B))
        x = to_dev(xb, shape.dtype)
        out = torch.zeros_like(x)
        tr = dl.trace_buffers(B)
        api.layer_forward(dl, x, out, ws, tr)
        torch.cuda.synchronize()
        worst = check_layer_trace(L, xb, tr, out)
        print("worst rel-L2 per stage:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
        # independent tokens really have different index sets
        if B > 1:
            i4 = tr["idx4"].cpu().numpy()
            assert not np.array_equal(i4[0], i4[1])


def test_config3_llama2_70b_layer_on_one_gpu(api):
    """LLaMA2-70B-shaped single layer, bf16, batch 1, 40 % sparsity, heavy-tailed (Student-t, nu=3)
    latent activations, PCA rotations (8192 x 8192) from 8192 synthetic calibration tokens."""
    shape = synth.SHAPES["llama2-70b"]
    print("building llama2-70b case (PCA at d=8192 on the host)", flush=True)
    case = cases.build_block_layer(shape, 0.4, seed=synth.seed_for(3, 0), n_cal=8192, latent="t3")
    assert (case.layer.K1, case.layer.K4) == (4915, 17203)
    print("running", flush=True)
    xb, out, tr, dl, ws = _run_layer(api, case, 1, seed=synth.seed_for(3, 5))
    worst = check_layer_trace(case.layer, xb, tr, out)
    print("worst rel-L2 per stage:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)


def test_config3_llama2_70b_shortcut_form_full_size(api):
    """The 70B-shaped layer in the form and launch shapes the bench times: rotations absorbed, two
    8192 x 8192 residual adapters that share the launches of q|k|v (adapter larger than the
    projection's kept rows: half of the workgroups each) and of gate|up (projection several times the
    adapter: three quarters of the workgroups), Top-K of the 28672-wide MLP vector in its own kernel.
    The two bases are seeded random orthogonal matrices (the attention one is the basis planted in the
    activation source, which PCA of such tokens recovers), so the host pays for the folds only."""
    shape = synth.SHAPES["llama2-70b"]
    seed = synth.seed_for(3, 0)
    print("building llama2-70b shortcut-form case (planted bases, fp64 folds on the host)", flush=True)
    bases = ([synth.planted_basis(shape.d, seed)], [synth.planted_basis(shape.d, seed + 7)])
    layers, bits, Qa, Ws, src = cases.build_shortcut_stack(shape, 1, 0.4, seed=seed, n_cal=0, bases=bases)
    L = layers[0]
    assert (L.K1, L.K2, L.K3, L.K4) == (4915, 4915, 4915, 17203)
    case = cases.LayerCase(shape, bits[0], L, {}, src)
    xb = O.encode16(O.rotate(src.draw(1, synth.seed_for(3, 5)), Qa[0]), shape.dtype)
    dl = device_layer(case)
    ws = api.Workspace(dl.workspace_bytes(1))
    x = to_dev(xb, shape.dtype)
    out = torch.zeros_like(x)
    tr = dl.trace_buffers(1)
    print("running", flush=True)
    api.layer_forward(dl, x, out, ws, tr)
    torch.cuda.synchronize()
    worst = check_layer_trace(L, xb, tr, out)
    print("worst rel-L2 per stage:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)


def test_config4_folded_stack_llama2_7b_shape(api):
    """Deployed form at LLaMA2-7B layer shape: rotations folded (no explicit Q), per-layer adapter as
    a dense 4096 x 4096 mat-vec; a 2-layer slice of the stack at batch 1, 8 and 32 (32 tokens fill the
    matrix-core kernel's two-tile token group), every stage of every layer and token checked.
    (The full 32-layer stack differs only in the number of such layers.)"""
    shape = synth.SHAPES["llama2-7b"]
    print("building 2 folded llama2-7b layers", flush=True)
    layers, bits, Qs, Ws, src = cases.build_folded_stack(shape, 2, 0.4, seed=synth.seed_for(4, 0), n_cal=4096)
    dls = [device_layer(cases.LayerCase(shape, b, L, {}, src)) for L, b in zip(layers, bits)]
    for B in (1, 8, 32):
        x0 = O.rotate(src.draw(B, seed=synth.seed_for(4, 5) + B), Qs[0])
        cur = to_dev(O.encode16(x0, shape.dtype), shape.dtype)
        for li, (L, dl) in enumerate(zip(layers, dls)):
            print(f"batch {B} layer {li}", flush=True)
            ws = api.Workspace(dl.workspace_bytes(B))
            out = torch.zeros_like(cur)
            tr = dl.trace_buffers(B)
            api.layer_forward(dl, cur, out, ws, tr)
            torch.cuda.synchronize()
            check_layer_trace(L, to_bits(cur), tr, out)
            cur = out
            del ws, tr


def test_config4_chain_of_layers_in_the_benchmarked_graph_form(api):
    """The form `bench.py --config 4` times: one rotation Q_l per layer, every rotation absorbed (q|k|v and
    gate|up carry Q_l^T, o carries Q_l, down carries Q_{l+1}), the residual adapter Q_l^T Q_{l+1} on the MLP
    shortcut only, at the LLaMA2-7B layer shape, batch 1.  A chain of 4 such layers, each layer's every stage
    checked against the oracle on the GPU's own input of that layer; then the same chain as ONE HIP graph,
    replayed with eager work in between, must reproduce the eager chain's output bits every time.
    The bases are seeded orthogonal matrices (any orthogonal matrices give a valid layer), so the host
    pays for the fp64 folds only."""
    shape = synth.SHAPES["llama2-7b"]
    n = 4
    seed = synth.seed_for(4, 0)
    Qs = [synth.planted_basis(shape.d, seed + 11 * l) for l in range(n)]
    print("building a 4-layer chain (fp64 folds on the host)", flush=True)
    layers, bits, Qa, Ws, src = cases.build_shortcut_stack(shape, n, 0.4, seed=seed, n_cal=0, bases=(Qs, Qs))
    for L, b in zip(layers, bits):      # Qa_l = Qm_l: the attention shortcut's adapter is the identity and is left out
        L.shortcut_attn = None
        b["shortcut_attn"] = None
    dls = [device_layer(cases.LayerCase(shape, b, L, {}, src)) for L, b in zip(layers, bits)]
    ws = api.Workspace(max(dl.workspace_bytes(1) for dl in dls))
    x0 = to_dev(O.encode16(O.rotate(src.draw(1, seed=synth.seed_for(4, 5)), Qs[0]), shape.dtype), shape.dtype)
    cur = x0
    outs = []
    for li, (L, dl) in enumerate(zip(layers, dls)):
        print(f"layer {li}", flush=True)
        out = torch.zeros_like(cur)
        tr = dl.trace_buffers(1)
        api.layer_forward(dl, cur, out, ws, tr)
        torch.cuda.synchronize()
        check_layer_trace(L, to_bits(cur), tr, out)
        outs.append(out)
        cur = out
    final_bits = to_bits(cur)
    # the chain as one graph (no trace buffers), as the bench builds it
    bufs = [torch.zeros_like(x0), torch.zeros_like(x0)]

    def chain():
        c = x0
        for i, dl in enumerate(dls):
            api.layer_forward(dl, c, bufs[i & 1], ws)
            c = bufs[i & 1]

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chain()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        chain()
    for rep in range(3):
        bufs[0].zero_(); bufs[1].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(to_bits(bufs[(n - 1) & 1]), final_bits), f"graph replay {rep}"
