"""The paper's iteration-time model as a calculator (host arithmetic only).

Symbols follow Table 1 and Sec. 2 of the SSD-SGD paper: T_f, T_b forward and
backward time of one iteration, T_c communication time of one iteration,
h_b_L backward time of the last layer, h_c_1 communication time of the first
layer, sum_h_s the total gradient-sending (Push) time, h_loc_1 local-update
time of the first layer, k the number of delay steps.
"""


def t_iter_ssgd(T_f, T_b, T_c, h_b_L, h_c_1, comm_bound):
    """Eq. (2): iteration time of SSGD.  comm_bound: the second case, backward
    time of layers 1..L-1 does not cover the communication of layers 2..L."""
    return T_f + T_c + h_b_L if comm_bound else T_f + T_b + h_c_1


def case_of(T_f, T_b, sum_h_s, h_loc_1):
    """Which case of Eq. (4) / Fig. 2 applies: 1 if the Push time is shorter
    than T_b + T_f + h_loc_1, else 2."""
    return 1 if sum_h_s < T_b + T_f + h_loc_1 else 2


def t_avg_k(k, T_f, T_b, T_c, h_b_L, sum_h_s, h_loc_1):
    """Eq. (4): average iteration time of SSD-SGD over k iterations (cases 1, 2)."""
    if case_of(T_f, T_b, sum_h_s, h_loc_1) == 1:
        return T_f + T_b + h_loc_1 + (T_c + h_b_L - T_f - 2 * T_b - h_loc_1) / k
    return sum_h_s + (T_c + h_b_L - T_b - sum_h_s) / k


def t_avg_compute_bound(T_f, T_b, h_loc_1):
    """Case 3 (text below Eq. (4)): computation dominates; independent of k."""
    return T_f + T_b + h_loc_1


def delta_t_k(k, T_f, T_b, T_c, h_b_L, h_loc_1, case):
    """Eq. (7): time saved over k iterations against SSGD, with the paper's
    simplification sum_h_s = T_c / 2 in case 2."""
    if case == 1:
        return (k - 1) * (T_c - T_b + h_b_L - h_loc_1) + (T_f + T_b)
    return k * T_f + (k - 1) / 2.0 * T_c + (k - 1) * h_b_L + T_b


def speedup_over_ssgd(k, T_f, T_b, T_c, h_b_L, sum_h_s, h_loc_1):
    """Training-speed gain of SSD-SGD over SSGD in the communication-bound
    regime, as the paper reports it (0.5 = 50 % faster)."""
    return t_iter_ssgd(T_f, T_b, T_c, h_b_L, 0.0, True) / t_avg_k(k, T_f, T_b, T_c, h_b_L, sum_h_s, h_loc_1) - 1.0
