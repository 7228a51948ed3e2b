"""The analytic runtime model (Section 3.1: Equations 1 and 2, Table 1) against what the paper
prints and against the table's own algebra."""
import os

import pytest

from paper_2502_02406_amd import runtime_model as M

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "comm_volume_video_mme.txt")


def test_volume_ratio_matches_the_printed_video_mme_figure():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    for sq, skv, d, pct in rows:
        ratio = M.volume_ratio(int(sq), int(skv), int(d)) * 100.0
        assert round(ratio, 2) == float(pct), ratio          # 0.0362 % rounds to the printed 0.04 %
        # the L term is what separates the ratio from S_Q / S_KV
        assert ratio == pytest.approx(int(sq) / int(skv) * (1 + 1 / (2 * int(d))) * 100.0, rel=1e-12)


def test_round_sizes_follow_equations_2_and_3():
    assert M.lvxattn_round_elements(10, 4) == 2 * 10 * 4 + 10
    assert M.ring_round_elements(1000, 4) == 2 * 1000 * 4
    assert M.lvxattn_round_elements(10, 4, h=3) == 3 * 90
    assert M.round_time(2.0, 100.0, 10.0) == 10.0              # transfer-bound
    assert M.round_time(2.0, 10.0, 10.0) == 2.0                # compute-bound: the transfer hides


def test_table1_speedup_is_the_ratio_of_its_two_rows():
    n, sq, skv, h, d = 8, 4096, 1 << 20, 32, 128
    flops, bw = 1.0e15, 2.0e9                                  # FLOP/s, elements/s
    for backward, ring_units, lv_units in ((False, 2, 4), (True, 4, 10)):
        ring = ring_units * (skv / n) * h * d / bw
        lv = lv_units * (sq / n) * (skv / n) * h * d / flops
        assert M.table1_speedup(sq // n, flops, bw, backward) == pytest.approx(ring / lv, rel=1e-12)


def test_prediction_for_the_bench_shape():
    # Sq = 2048 against a block of 32768 keys, 32 / 8 heads of 128, 0.9 ms per visit
    p = M.predict_forward_round(0.9, 2048, 32768, 128, 32, 8, "link", 100.0)
    assert p.lvxattn_comm_ms == pytest.approx(32 * (2048 * 128 * 6 + 2048 * 4) / 100e9 * 1e3)
    assert p.ring_comm_ms == pytest.approx(8 * 2 * 32768 * 128 * 2 / 100e9 * 1e3)
    assert p.lvxattn_hidden and p.lvxattn_round_ms == pytest.approx(0.9)
    assert p.ring_round_ms == pytest.approx(max(0.9, p.ring_comm_ms))
    slow = M.predict_forward_round(0.9, 2048, 32768, 128, 32, 8, "nic", 1.25)
    assert not slow.lvxattn_hidden and slow.speedup == pytest.approx(slow.ring_comm_ms / slow.lvxattn_comm_ms)


def test_backward_prediction_counts_the_travelling_tensors():
    p = M.predict_backward_round(2.8, 2048, 32768, 128, 32, 8, "link", 153.0)
    assert p.lvxattn_comm_ms == pytest.approx(32 * (2048 * 128 * 8 + 2 * 2048 * 4) / 153e9 * 1e3)
    assert p.ring_comm_ms == pytest.approx(8 * 2 * 32768 * 128 * 6 / 153e9 * 1e3)
    assert p.lvxattn_hidden and p.lvxattn_round_ms == pytest.approx(2.8)
    # with equal element sizes the ratio of the two volumes is Table 1's: 4 units of S_KV against
    # the query side's 3 tensors of S_Q (plus the statistics)
    q = M.predict_backward_round(1e-9, 100, 5000, 64, 4, 4, "x", 1.0, 2, 2, 2, 2, 2, 2)
    assert q.ring_comm_ms / q.lvxattn_comm_ms == pytest.approx(4 * 5000 * 64 / (3 * 100 * 64 + 2 * 100))
