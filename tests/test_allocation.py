"""Kept-count allocation across h1..h4 (App. B): the product-side bookkeeping against the oracle's
statement of the constraints and the coefficients the paper prints."""
import os

from oracle import larosa_oracle as O
from paper_2507_01299_amd import allocation

GOLD = os.path.join(os.path.dirname(__file__), "golden", "table11_alpha.txt")
DIMS = {"LLaMA2-7B": (4096, 4096, 4096, 11008), "LLaMA3-8B": (4096, 4096, 1024, 14336),
        "LLaMA2-70B": (8192, 8192, 1024, 28672), "LLaMA3-70B": (8192, 8192, 1024, 28672),
        "Mistral-7B": (4096, 4096, 1024, 14336), "Qwen2.5-7B": (3584, 3584, 512, 18944)}


def rows():
    with open(GOLD) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                m, a1, a2, a3, a4, M = line.split()
                yield m, float(a1), float(a2), float(a3), float(a4), float(M)


def test_uniform_alpha_gives_the_benchmark_counts():
    assert allocation.kept_counts(4096, 4096, 11008, 0.4) == (2457, 2457, 2457, 6604)
    assert allocation.kept_counts(4096, 4096, 14336, 0.25) == (3072, 3072, 3072, 10752)
    assert allocation.kept_counts(8192, 8192, 28672, 0.4) == (4915, 4915, 4915, 17203)


def test_printed_coefficients_give_oracle_counts_and_keep_the_block_totals():
    for model, a1, a2, a3, a4, M in rows():
        d, d_q, d_kv, d_ff = DIMS[model]
        assert abs(d_ff / d - M) < 1e-3
        for p in (0.25, 0.4, 0.5):
            Ks = allocation.kept_counts(d, d_q, d_ff, p, a1, a3)
            want = (O.kept_count(d, p, a1), O.kept_count(d_q, p, O.alpha_partner_attn(a1)),
                    O.kept_count(d, p, a3), O.kept_count(d_ff, p, O.alpha_partner_mlp(a3, d_ff / d)))
            assert Ks == want, (model, p)
            if max(4 - 3 * a1, (2 + M - 2 * a3) / M) * (1 - p) <= 1.0:      # no clamping at the width
                # kept activation entries per block, each counted once per projection it feeds
                attn = 3 * Ks[0] + Ks[1]
                mlp = 2 * Ks[2] + Ks[3]
                assert abs(attn - 4 * (1 - p) * d) <= 4
                assert abs(mlp - (2 + M) * (1 - p) * d) <= 4


def test_allocation_moves_weight_bytes_at_fixed_sparsity():
    d, d_q, d_kv, d_ff = DIMS["LLaMA2-7B"]
    uni = allocation.selected_weight_bytes(d, d_q, d_kv, d_ff, allocation.kept_counts(d, d_q, d_ff, 0.4))
    gs = allocation.selected_weight_bytes(d, d_q, d_kv, d_ff, allocation.kept_counts(d, d_q, d_ff, 0.4, 0.90, 0.80))
    assert uni == 242797568
    assert 0.90 * uni < gs < uni        # fewer gate|up rows outweigh more down rows
