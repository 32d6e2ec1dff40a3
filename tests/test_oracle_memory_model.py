"""The activation-memory model against the numbers the paper prints (Sec. 2.1; App. E.3; App. H)."""
import json
import os

import pytest

from oracle import tempo_oracle as O

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


@pytest.mark.parametrize("S", [128, 512, 2048])
def test_ablation_percentages(S):
    g = GOLD["ablation_percent"]
    H, A, e = 1024, 16, 4            # H/A = 64, 32-bit activations
    total = O.activation_bytes_baseline(H, A, S, e)
    saved = O.activation_bytes_saved_paper(H, A, S, e)
    got = [round(100.0 * saved[k] / total, 2) for k in g["order"]]
    assert got == g[str(S)]
    # the ratio H/A fixes the percentages, not H itself
    total2 = O.activation_bytes_baseline(768, 12, S, e)
    saved2 = O.activation_bytes_saved_paper(768, 12, S, e)
    assert [round(100.0 * saved2[k] / total2, 2) for k in g["order"]] == g[str(S)]


def test_attention_maps_share():
    g = GOLD["attention_maps_share_bert_base_s512"]
    total = O.activation_bytes_baseline(g["H"], g["A"], g["S"], 4)
    three_maps = 3 * g["A"] * g["S"] * 4
    assert int(100.0 * three_maps / total) == g["value"]


def test_gelu_input_share():
    g = GOLD["gelu_input_share_bert_base_s128"]
    total = O.activation_bytes_baseline(g["H"], g["A"], g["S"], 4)
    share = 100.0 * (4 * g["H"] * 4) / total
    assert g["value"] <= share < g["value"] + 0.5      # "almost 17 %"


def test_byte_mask_fraction():
    # discarding an fp32 dropout output while keeping its byte mask saves 4/5 of (output + mask)
    A, S = 12, 512
    out_bytes, mask_bytes = A * S * 4, A * S
    assert out_bytes / (out_bytes + mask_bytes) == GOLD["byte_mask_saving_fraction"]["value"]
    assert O.activation_bytes_saved_paper(768, A, S, 4)["dropout"] == out_bytes


def test_bitmask_savings_exceed_byte_mask_savings():
    for (H, A, S, e) in [(768, 12, 128, 4), (1024, 16, 128, 2), (1024, 16, 512, 2), (768, 12, 1024, 2)]:
        a = O.activation_bytes_saved_paper(H, A, S, e)
        b = O.activation_bytes_saved_bitmask(H, A, S, e)
        assert all(b[k] >= a[k] for k in a)
    # worked totals: fp32 BERT-base S=128 and bf16 BERT-large S=512
    assert sum(O.activation_bytes_saved_bitmask(768, 12, 128, 4).values()) == 31688
    assert O.activation_bytes_baseline(768, 12, 128, 4) == 70656
    assert sum(O.activation_bytes_saved_bitmask(1024, 16, 512, 2).values()) == 51720
    assert O.activation_bytes_baseline(1024, 16, 512, 2) == 92160
