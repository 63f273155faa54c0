"""The operation / byte counts the benchmark reports against (Sec. 3.4 of arxiv 2508.10395), pinned to the two
context lengths the paper prints for its worked example."""
import os

import pytest

from paper_2508_10395_amd import cost_model as cm

GOLD = os.path.join(os.path.dirname(__file__), "golden", "cost_model.txt")
P_PAPER = 756e12 / 2e12          # the ridge point the section assumes
D = 4096


def _golden():
    rows = {}
    with open(GOLD) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, g, _, val = line.split()
                rows[name] = (int(g), float(val))
    return rows


def test_ridge_point_of_the_worked_example():
    assert P_PAPER == 378.0


def test_max_remat_tokens_llama2_7b_printed_value():
    g, printed_k = _golden()["llama2_7b"]
    l = cm.max_remat_tokens(P_PAPER, D, 2, cm.layer_weight_bytes_llama2_7b(D), g)
    assert round(l) == 2281
    assert round(l / 1000.0, 1) == printed_k
    # it solves the section's equation
    assert cm.remat_flops(l, D) / (cm.x_cache_bytes(l, D, 2) + cm.layer_weight_bytes_llama2_7b(D)) == pytest.approx(P_PAPER, rel=1e-12)


def test_max_remat_tokens_llama31_8b_printed_value():
    g, printed_k = _golden()["llama31_8b"]
    wb = cm.layer_weight_bytes_llama31_8b(D, g)
    l = cm.max_remat_tokens(P_PAPER, D, 2, wb, g)
    assert round(l) == 40627
    assert round(l / 1000.0, 1) == printed_k
    assert cm.remat_flops(l, D, g) / (cm.x_cache_bytes(l, D, 2, g) + wb) == pytest.approx(P_PAPER, rel=1e-12)
    # the running text's byte count (twice the equation's) would not reproduce the printed value
    l_text = P_PAPER * wb / (4.0 * (D / g) ** 2 - P_PAPER * cm.kv_cache_bytes(1, D, 2, g))
    assert round(l_text / 1000.0, 1) != printed_k


def test_counts_of_the_section():
    l = 1000
    assert cm.remat_flops(l, D) == 4.0 * l * D * D
    assert cm.remat_flops(l, D, 4) == cm.remat_flops(l, D) / 16          # g^2 fewer operations
    assert cm.x_cache_bytes(l, D, 3) == 3 / 8 * l * D
    assert cm.kv_cache_bytes(l, D, 3) == 2 * cm.x_cache_bytes(l, D, 3)   # X is one tensor, K and V are two
    assert cm.remat_flops(l, D) + cm.cl_extra_flops(l, D) == pytest.approx(4.0 * l * D * (D + 0.5))
    assert cm.cl_gqa_flops(l, D, 4) == 8.0 * l * (D / 4) * D


def test_launch_counts_reduce_to_the_section_for_mha():
    """The benchmark's per-launch FLOPs: for MHA (n_kv_heads * head_dim = d) the contraction term is the
    section's 2*2*l*d^2 summed over the batch; config 2 gives the 2.1996e12 quoted with its roofline."""
    B, L, Hq, hd = 8, 4096, 32, 128
    total = cm.remat_attn_flops(B * L, D, Hq, Hq, hd)
    assert total - 4.0 * B * L * Hq * hd == B * cm.remat_flops(L, D)
    assert total == pytest.approx(2.1996e12, rel=1e-4)
    # algorithmic bytes of the same launch: 3-bit codes 50.3 MB + metadata 4.2 MB + weights 67.1 MB
    by = cm.remat_attn_algorithmic_bytes(B * L, D, 3, 128, Hq, hd)
    assert by == pytest.approx(50.33e6 + 4.19e6 + 67.11e6, rel=1e-3)
    assert cm.quantize_bytes_per_element(3, 128) == 2 + 3 / 8 + 4 / 128
    assert cm.cl_accumulate_bytes_per_element(2, 128) == cm.quantize_bytes_per_element(2, 128, True)
