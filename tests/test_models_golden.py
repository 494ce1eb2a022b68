"""The byte and flop models against the values the paper prints (Tables 1 and 2)."""
import os

import pytest

from paper_2603_02188_amd import roofline as rf
from paper_2603_02188_amd.inputs import WORKLOADS, draw_seq_lens

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_table1_kv_loading_per_device():
    d_h = 128
    for method, *vals in _rows("table1_kv_loading.txt"):
        for tp, want in zip((1, 2, 4, 8), vals):
            got = rf.kv_loading_per_token(method, tp, d_h=d_h, h=64, g=8) / d_h
            assert got == pytest.approx(float(want), abs=1e-12), (method, tp)


def test_table2_arithmetic_intensity_limits():
    h, g, d_h = 128, 8, 128
    approx = {"1": 1.0, "h": float(h), "h/g": h / g, "2h": 2.0 * h}
    for method, sym in _rows("table2_arithmetic_intensity.txt"):
        exact = rf.arithmetic_intensity(method, h=h, d_h=d_h, g=g)
        # Table 2's second row drops the RoPE terms; the exact ratio sits within 20 % below it.
        assert 0.8 * approx[sym] <= exact <= approx[sym] + 1e-9, (method, exact)
    # Table 2's closed form for MLRA-4 at the bench shapes: (4 h d_c/4 + 2 h d_r) / (2 (d_c/4 + d_r)).
    assert rf.arithmetic_intensity("MLRA-4", h=128, d_h=128) == pytest.approx((65536 + 16384) / 384.0)
    assert rf.arithmetic_intensity("MLA", h=128, d_h=128) == pytest.approx((262144 + 16384) / 1152.0)


def test_workload_bytes_follow_table1():
    """Cache bytes per token of the bench workloads are Table 1's per-device element counts x 2 B."""
    c2, c3 = WORKLOADS["C2"], WORKLOADS["C3"]
    b2 = rf.decode_bytes(draw_seq_lens(c2), c2.h, c2.d_h, c2.n_blocks, c2.d_cb, c2.d_r)
    b3 = rf.decode_bytes(draw_seq_lens(c3), c3.h, c3.d_h, c3.n_blocks, c3.d_cb, c3.d_r)
    assert b2["tokens"] == 16 * 16384 and b3["tokens"] == 64 * 8192
    assert b2["cache"] == b2["tokens"] * 2 * rf.kv_loading_per_token("MLRA-4", 4, d_h=128)   # 1.5 d_h
    assert b3["cache"] == b3["tokens"] * 2 * rf.kv_loading_per_token("MLRA-4", 1, d_h=128)   # 4.5 d_h
    assert b2["total"] == pytest.approx(106.2e6, rel=2e-3) and b3["total"] == pytest.approx(632.3e6, rel=2e-3)
    f3 = rf.decode_flops(draw_seq_lens(c3), c3.h, c3.d_h, c3.n_blocks, c3.d_cb, c3.d_r)
    # Step 2 alone is Table 2's numerator per block times four blocks.
    step2 = 64 * 8192 * 4 * (4 * 128 * 128 + 2 * 128 * 64)
    assert f3 == pytest.approx(step2 + 64 * 128 * 2 * 512 * 128)
