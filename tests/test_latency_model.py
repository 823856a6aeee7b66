"""The M/D/1 latency model of the paper's Section "Streaming inference" against closed forms."""
import math

import pytest

from paper_2311_04996_amd.latency_model import load_table, total_latency


def test_idle_server_has_no_queue():
    assert total_latency(0.010, 0.0) == pytest.approx(0.010)


def test_half_load_waits_half_a_service_time():
    # rho = 1/2: queue term = lam / (2 mu (mu - lam)) = (mu/2) / (2 mu (mu/2)) = D / 2
    D = 0.020
    assert total_latency(D, 0.5 / D) == pytest.approx(1.5 * D)


def test_matches_pollaczek_khinchine_for_constant_service():
    # M/G/1: W_q = lam E[S^2] / (2 (1 - rho)); constant service: E[S^2] = D^2
    D = 0.0137
    for rho in (0.1, 0.3, 0.77, 0.95):
        lam = rho / D
        assert total_latency(D, lam) == pytest.approx(D + lam * D * D / (2.0 * (1.0 - rho)))


def test_saturated_and_invalid():
    assert math.isinf(total_latency(0.01, 100.0))
    assert math.isinf(total_latency(0.01, 250.0))
    with pytest.raises(ValueError):
        total_latency(0.0, 1.0)
    with pytest.raises(ValueError):
        total_latency(0.01, -1.0)


def test_halving_latency_cuts_queue_time_more_than_fourfold_at_fixed_arrivals():
    # the paper's point: wait time falls quadratically (and more) with the serving rate
    lam = 40.0
    q1 = total_latency(0.020, lam) - 0.020
    q2 = total_latency(0.010, lam) - 0.010
    assert q2 < q1 / 4.0


def test_load_table_rows():
    rows = load_table(0.010, 0.64, 512, loads=(0.5,))
    assert rows[0]["streams_at_realtime"] == int(0.5 / 0.010 * 0.64 * 512)
    assert rows[0]["total_ms"] == pytest.approx(15.0)
    assert rows[0]["queue_ms"] == pytest.approx(5.0)
