"""The flop counter reproduces the layer-level FLOP table the paper prints (App. G) and its
complexity model (App. C)."""
import os

import pytest

from paper_2509_10918_amd import costs

GOLD = os.path.join(os.path.dirname(__file__), "golden", "flop_table.txt")


def _rows():
    with open(GOLD) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                m, seq, dim, orig, toma, ovh = line.split()
                yield m, int(seq), int(dim), float(orig), float(toma), float(ovh)


def test_flop_table():
    for model, seq, dim, orig, toma, ovh in _rows():
        B = 1 if model == "flux" else 2           # SDXL runs a classifier-free-guidance pair
        text = 512 if model == "flux" else 0      # Flux: 4096 image + 512 text tokens
        n_img = seq - text
        assert costs.attention_block_flops(B, seq, dim) / 1e9 == pytest.approx(orig, rel=0.03)
        merged = n_img // 2 + text                # text tokens stay unmerged
        assert costs.attention_block_flops(B, merged, dim) / 1e9 == pytest.approx(toma, rel=0.03, abs=0.5)
        # overhead with 256 regions and region-local merge
        n_loc = n_img // 256
        o = costs.toma_overhead_flops(B, n_img, dim, n_loc, n_loc // 2) / 1e9
        assert o == pytest.approx(ovh, abs=0.011)


def test_complexity_model_terms():
    # App. C per sample, one region: C_sub = N^2 d, C_proj = C_merge = C_unmerge = N D d
    N, D, d = 4096, 2048, 640
    s = costs.stage_flops(1, N, d, 1, D, 1)
    assert s["similarity"] == 2 * N * N * d
    assert s["weights"] == s["merge"] == s["unmerge"] == 2 * N * D * d
    # k regions: selection cost / k, weights and (un)merge / k^2 per region => / k in total
    k = 16
    sk = costs.stage_flops(1, N, d, k, D // k, k)
    assert sk["similarity"] * k == s["similarity"]
    assert sk["merge"] * k == s["merge"]
    assert costs.greedy_stream_bytes(2, 16, 256, 128) == 1065353216
