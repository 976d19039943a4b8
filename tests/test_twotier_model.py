"""The host-side byte/latency model against the dense throughputs the paper prints."""
import json
import os

import pytest

from paper_2412_01380_amd.twotier import (Device, dense_tokens_per_second, sparse_tokens_per_second,
                                          token_seconds)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "dense_throughput_tables.json")


def test_dense_rows_of_the_paper_tables():
    g = json.load(open(GOLDEN))
    for row in g["phi3_medium_exact"]:
        got = dense_tokens_per_second(row["model_gb"] * 1e9, row["dram_gb"] * 1e9,
                                      Device(flash_gbps=row["flash_gbps"]))
        assert round(got, 2) == row["tok_s"], row["source"]
    # sizes printed to 0.1 GB leave up to ~6 % slack on the small models
    for row in g["other_models_rounded_sizes"]:
        got = dense_tokens_per_second(row["model_gb"] * 1e9, row["dram_gb"] * 1e9,
                                      Device(flash_gbps=row["flash_gbps"]))
        assert got == pytest.approx(row["tok_s"], rel=0.06), row["source"]


def test_additive_variant_and_limits():
    d = Device()
    assert token_seconds(1e9, 6e9, d, overlap=False) == pytest.approx(1.0 + 0.1)
    assert token_seconds(1e9, 6e9, d, overlap=True) == pytest.approx(1.0)
    # everything resident: DRAM-bound
    assert dense_tokens_per_second(3e9, 4e9, d) == pytest.approx(60.0 / 3.0)


def test_sparse_model_is_monotone_in_hit_rate_and_density():
    kw = dict(static_bytes=1e9, layers=40, col_bytes_in=18480.0, col_bytes_mid=2640.0)
    lo = sparse_tokens_per_second(selected_in=1536, selected_mid=5376, hit_rate_in=0.5, hit_rate_mid=0.5, **kw)
    hi = sparse_tokens_per_second(selected_in=1536, selected_mid=5376, hit_rate_in=0.9, hit_rate_mid=0.9, **kw)
    dn = sparse_tokens_per_second(selected_in=2560, selected_mid=8960, hit_rate_in=0.5, hit_rate_mid=0.5, **kw)
    assert hi > lo > dn
    # closed form at one operating point: misses = 40*(768*18480 + 2688*2640) bytes at 1 GB/s
    miss = 40 * (768 * 18480 + 2688 * 2640)
    assert lo == pytest.approx(1.0 / (miss / 1e9))
