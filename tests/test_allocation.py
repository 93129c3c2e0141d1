"""Kept-count allocation across h1..h4 (App. B): the product-side bookkeeping against counts worked out
by hand from the paper's printed coefficients and constraints (tests/golden/appendix_b_kept_counts.txt),
and against the constraints themselves.  The oracle's own kept_count is held to the same fixture, so the
two sides are each pinned to the paper, not to each other."""
import os

from oracle import larosa_oracle as O
from paper_2507_01299_amd import allocation

GOLD = os.path.join(os.path.dirname(__file__), "golden")
DIMS = {"LLaMA2-7B": (4096, 4096, 4096, 11008), "LLaMA3-8B": (4096, 4096, 1024, 14336),
        "LLaMA2-70B": (8192, 8192, 1024, 28672), "LLaMA3-70B": (8192, 8192, 1024, 28672),
        "Mistral-7B": (4096, 4096, 1024, 14336), "Qwen2.5-7B": (3584, 3584, 512, 18944)}


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                yield line.split()


def test_uniform_alpha_gives_the_benchmark_counts():
    # the K values of the benchmark configurations: (1 - p) D truncated (0.6 * 4096 = 2457.6, 0.6 * 11008 = 6604.8, ...)
    assert allocation.kept_counts(4096, 4096, 11008, 0.4) == (2457, 2457, 2457, 6604)
    assert allocation.kept_counts(4096, 4096, 14336, 0.25) == (3072, 3072, 3072, 10752)
    assert allocation.kept_counts(4096, 4096, 14336, 0.5) == (2048, 2048, 2048, 7168)
    assert allocation.kept_counts(8192, 8192, 28672, 0.4) == (4915, 4915, 4915, 17203)
    assert allocation.kept_counts(512, 512, 1024, 0.5) == (256, 256, 256, 512)


def test_counts_from_the_printed_coefficients_match_the_hand_computed_fixture():
    n = 0
    for model, p, a1, a3, K1, K2, K3, K4 in _rows("appendix_b_kept_counts.txt"):
        d, d_q, d_kv, d_ff = DIMS[model]
        want = (int(K1), int(K2), int(K3), int(K4))
        assert allocation.kept_counts(d, d_q, d_ff, p, a1, a3) == want, (model, p)              # decimal strings
        assert allocation.kept_counts(d, d_q, d_ff, float(p), float(a1), float(a3)) == want, (model, p)
        n += 1
    assert n == 18


def test_oracle_kept_count_matches_the_same_fixture():
    for model, p, a1, a3, K1, K2, K3, K4 in _rows("appendix_b_kept_counts.txt"):
        d, d_q, d_kv, d_ff = DIMS[model]
        p, a1, a3 = float(p), float(a1), float(a3)
        got = (O.kept_count(d, p, a1), O.kept_count(d_q, p, O.alpha_partner_attn(a1)), O.kept_count(d, p, a3),
               O.kept_count(d_ff, p, O.alpha_partner_mlp(a3, d_ff / d)))
        assert got == (int(K1), int(K2), int(K3), int(K4)), (model, p)


def test_printed_table_satisfies_the_block_constraints_and_the_counts_keep_the_block_totals():
    for model, a1, a2, a3, a4, M in _rows("table11_alpha.txt"):
        a1, a2, a3, a4, M = map(float, (a1, a2, a3, a4, M))
        d, d_q, d_kv, d_ff = DIMS[model]
        assert abs(d_ff / d - M) < 1e-3
        assert abs(3 * a1 + a2 - 4) < 1e-9, model                  # attention block, printed exactly
        assert abs(2 * a3 + M * a4 - (2 + M)) <= 0.01 * M + 1e-9, model   # MLP block: alpha_4 is printed to 2 decimals
        #                                                                   (within one unit of the last place)
        for p in (0.25, 0.4, 0.5):
            Ks = allocation.kept_counts(d, d_q, d_ff, p, a1, a3)
            if max(a2, (2 + M - 2 * a3) / M) * (1 - p) <= 1.0:      # no clamping at the width
                # kept activation entries per block, each counted once per projection it feeds
                assert abs(3 * Ks[0] + Ks[1] - 4 * (1 - p) * d) <= 4
                assert abs(2 * Ks[2] + Ks[3] - (2 + M) * (1 - p) * d) <= 4


def test_counts_are_clamped_to_the_width_and_to_one():
    assert allocation.kept_counts(4096, 4096, 11008, 0.25, 0.80, 0.80)[1] == 4096      # alpha_2 = 1.6: 1.2 D -> D
    assert allocation.kept_counts(64, 64, 128, 0.999) == (1, 1, 1, 1)


def test_allocation_moves_weight_bytes_at_fixed_sparsity():
    d, d_q, d_kv, d_ff = DIMS["LLaMA2-7B"]
    uni = allocation.selected_weight_bytes(d, d_q, d_kv, d_ff, allocation.kept_counts(d, d_q, d_ff, 0.4))
    gs = allocation.selected_weight_bytes(d, d_q, d_kv, d_ff, allocation.kept_counts(d, d_q, d_ff, 0.4, 0.90, 0.80))
    assert uni == 242797568
    assert 0.90 * uni < gs < uni        # fewer gate|up rows outweigh more down rows
