"""The timing-model calculator against the paper's own algebra: Eq. (7) is
printed independently of Eqs. (2) and (4) and must equal k*T_iter - k*T_avg,k."""
import itertools

import pytest

from paper_2012_05396_amd import timing_model as tm


@pytest.mark.parametrize("k", [2, 3, 5, 8])
def test_eq7_equals_k_times_eq2_minus_eq4_case1(k):
    for T_f, T_b, T_c, h_b_L, h_loc in itertools.product((1.0, 2.5), (2.0, 4.0), (20.0, 33.0), (0.3,), (0.2, 0.7)):
        sum_h_s = 0.5 * (T_b + T_f + h_loc)          # case 1: Push shorter than compute
        assert tm.case_of(T_f, T_b, sum_h_s, h_loc) == 1
        lhs = k * tm.t_iter_ssgd(T_f, T_b, T_c, h_b_L, 0.0, True) - k * tm.t_avg_k(k, T_f, T_b, T_c, h_b_L, sum_h_s, h_loc)
        assert lhs == pytest.approx(tm.delta_t_k(k, T_f, T_b, T_c, h_b_L, h_loc, 1), rel=1e-12)


@pytest.mark.parametrize("k", [2, 3, 5, 8])
def test_eq7_equals_k_times_eq2_minus_eq4_case2(k):
    for T_f, T_b, T_c, h_b_L, h_loc in itertools.product((1.0, 2.5), (2.0, 4.0), (20.0, 33.0), (0.3,), (0.2,)):
        sum_h_s = T_c / 2                            # the paper's simplification for Eq. (7)
        assert tm.case_of(T_f, T_b, sum_h_s, h_loc) == 2
        lhs = k * tm.t_iter_ssgd(T_f, T_b, T_c, h_b_L, 0.0, True) - k * tm.t_avg_k(k, T_f, T_b, T_c, h_b_L, sum_h_s, h_loc)
        assert lhs == pytest.approx(tm.delta_t_k(k, T_f, T_b, T_c, h_b_L, h_loc, 2), rel=1e-12)


def test_larger_k_is_faster_in_both_cases():
    """Sec. 2.2: the bracket of Eq. (4) is positive, so T_avg,k falls with k."""
    a = [tm.t_avg_k(k, 1.0, 2.0, 20.0, 0.3, 1.0, 0.2) for k in (2, 3, 4, 8)]
    b = [tm.t_avg_k(k, 1.0, 2.0, 20.0, 0.3, 10.0, 0.2) for k in (2, 3, 4, 8)]
    assert a == sorted(a, reverse=True) and b == sorted(b, reverse=True)
    assert tm.speedup_over_ssgd(5, 1.0, 2.0, 20.0, 0.3, 10.0, 0.2) > tm.speedup_over_ssgd(2, 1.0, 2.0, 20.0, 0.3, 10.0, 0.2) > 0


def test_hand_evaluated_values():
    # T_f=1, T_b=2, T_c=20, h_b_L=0.5, sum_h_s=1 (<3.2: case 1), h_loc=0.2, k=4
    assert tm.t_iter_ssgd(1, 2, 20, 0.5, 0.0, True) == 21.5
    assert tm.t_avg_k(4, 1, 2, 20, 0.5, 1, 0.2) == pytest.approx(3.2 + (20.5 - 1 - 4 - 0.2) / 4)
    assert tm.t_iter_ssgd(1, 2, 20, 0.5, 0.7, False) == 3.7
    assert tm.t_avg_compute_bound(1, 2, 0.2) == 3.2
