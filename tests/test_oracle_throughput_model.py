"""Pins for the throughput model (Section "Throughput-Guided Hybrid Coordination", eqs. thr_ordinary,
thr_parallel, r_threshold; Appendix "Detailed Throughput Analysis")."""
import math


def test_threshold_is_where_the_two_throughputs_cross(oracle):
    for (B, L, gamma, T_D, T_T) in [(32, 2.6, 4, 3.0, 40.0), (128, 3.6, 4, 1.0, 47.0), (64, 1.5, 8, 2.0, 30.0)]:
        assert gamma * T_D < T_T
        rs = oracle.r_star(L, gamma, T_D, T_T)
        assert math.isclose(oracle.thr_ordinary(B, L, gamma, T_D, T_T), oracle.thr_parallel(B, L, rs, T_T), rel_tol=1e-12)
        assert oracle.thr_parallel(B, L, rs * 0.9, T_T) > oracle.thr_ordinary(B, L, gamma, T_D, T_T)
        assert oracle.thr_parallel(B, L, min(1.0, rs * 1.1), T_T) < oracle.thr_ordinary(B, L, gamma, T_D, T_T)


def test_hand_worked_value(oracle):
    # gamma = 4, L = 3, T_D = 1, T_T = 10: r* = 3*3*1 / ((10+3)*2) = 9/26
    assert math.isclose(oracle.r_star(3.0, 4.0, 1.0, 10.0), 9.0 / 26.0, rel_tol=1e-15)
    # all requests fall back (r = 1): parallel mode is autoregressive, B tokens per T_T
    assert oracle.thr_parallel(32, 3.0, 1.0, 10.0) == 3.2
    # no fallback: B*L per T_T
    assert oracle.thr_parallel(32, 3.0, 0.0, 10.0) == 9.6
