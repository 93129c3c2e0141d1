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


@pytest.fixture(params=[(1, 8), (1, 16), (0, 8)], ids=["fused8", "fused16", "separate"])
def fused_mode(api, request):
    """Run the layer with the Top-K fused into the projection kernels (512- and 1024-lane
    workgroups) and as separate kernels."""
    api.set_tuning(3, request.param[0])
    api.set_tuning(4, request.param[1])
    yield request.param
    api.set_tuning(3, 1)
    api.set_tuning(4, 8)


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


def test_ragged_layer_shapes(api, fused_mode):
    """Widths that are not multiples of the 512-column strip or of the per-lane element run, GQA
    with 4 query heads per value head, K values at both extremes."""
    shape = synth.LayerShape("ragged", 328, 384, 96, 1000, 24, "bf16")
    for Ks in ((1, 384, 327, 999), (328, 1, 1, 1), (200, 100, 150, 613)):
        case = cases.build_block_layer(shape, 0.4, seed=71, n_cal=768, Ks=Ks)
        xb, out, tr, dl, ws = _run_layer(api, case, 2, seed=4)
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
