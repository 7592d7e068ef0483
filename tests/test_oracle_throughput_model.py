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


def test_next_mode_picks_the_faster_coordination(oracle):
    # eq. mode_switch_batch against the two throughput formulas it was derived from: PARALLEL iff it is
    # not slower at the observed rollback ratio (ties go to PARALLEL, as r_hat <= r* does)
    for (gamma, T_D, T_T) in [(4, 3.0, 40.0), (4, 1.0, 47.0), (8, 2.0, 30.0), (2, 5.0, 11.0)]:
        for B in (1, 7, 32, 256):
            for emitted in sorted({B, B + 1, 2 * B, int(2.6 * B), int(gamma * B)}):
                for R in sorted({0, 1 % (B + 1), B // 4, B // 2, B}):
                    mode, r_hat, r_star = oracle.next_mode(R, emitted, B, gamma, T_D, T_T)
                    L = emitted / B
                    assert r_hat == R / B
                    par, ordi = oracle.thr_parallel(B, L, R / B, T_T), oracle.thr_ordinary(B, L, gamma, T_D, T_T)
                    if not math.isclose(par, ordi, rel_tol=1e-12):
                        assert mode == (1 if par > ordi else 0), (gamma, T_D, T_T, B, emitted, R)
                    if L > 1:
                        assert math.isclose(r_star, oracle.r_star(L, gamma, T_D, T_T), rel_tol=1e-15)
                    else:
                        assert r_star == math.inf and mode == 1


def test_next_mode_hand_worked(oracle):
    # gamma = 4, T_D = 1, T_T = 10, B = 26, 78 tokens emitted (L = 3): r* = 9/26, so 9 rollbacks still run
    # PARALLEL and 10 switch to ORDINARY
    assert oracle.next_mode(9, 78, 26, 4, 1.0, 10.0)[0] == 1
    assert oracle.next_mode(10, 78, 26, 4, 1.0, 10.0)[0] == 0
