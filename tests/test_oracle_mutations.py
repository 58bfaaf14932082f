"""Do the pins bite?  Each plausible mistake below is planted in a copy of the
oracle's C source (on the CPU, in a temporary directory), the copy is built,
and the pins of test_oracle_pins.py are run against it: every mutant must fail
at least one pin.  The real oracle is restored afterwards."""
import ctypes
import os
import subprocess

import pytest

import oracle.ssd_oracle as O
from oracle import build as obuild

import test_oracle_pins as pins

MUTATIONS = {
    "momentum sign":            ("REAL mo = t4 - t3;", "REAL mo = t4 + t3;"),
    "weight decay dropped":     ("REAL t2 = gh + t1;", "REAL t2 = gh;"),
    "weight step sign":         ("w[j] = w[j] + mo;", "w[j] = w[j] - mo;"),
    "a worker left out":        ("for (int i = 1; i < K; ++i)\n            S = S + g[i][j];",
                                 "for (int i = 2; i < K; ++i)\n            S = S + g[i][j];"),
    "sum not averaged":         ("REAL gh = S * rescale;", "REAL gh = S;"),
    "momentum factor dropped":  ("REAL t4 = m * mom[j];", "REAL t4 = mom[j];"),
    "lr dropped in server":     ("REAL t3 = lr * t2;", "REAL t3 = t2;"),
    "grad_sync sign":           ("REAL e = q - wl[j];", "REAL e = wl[j] - q;"),
    "ascent as printed":        ("wl[j] = wl[j] - u6;", "wl[j] = wl[j] + u6;"),
    "beta dropped":             ("REAL u4 = beta * gs;", "REAL u4 = gs;"),
    "alpha dropped":            ("REAL u1 = alpha * g[j];", "REAL u1 = g[j];"),
    "local decay dropped":      ("REAL u2 = wd_loc * wl[j];", "REAL u2 = 0;"),
    "lr_loc dropped":           ("REAL u6 = lr_loc * u5;", "REAL u6 = u5;"),
    "refresh one step late":    ("int refresh = (lu > 0) && (lu % k == 0);",
                                 "int refresh = (lu > 0) && (lu % k == 1 % k) && (lu > 1 || k == 1);"),
    "refresh every step":       ("int refresh = (lu > 0) && (lu % k == 0);", "int refresh = (lu > 0);"),
    "pre_weight not initialised": ("        if (lu == 0)\n            pre[j] = wl[j];", "        ;"),
    "refresh takes updated w'": ("        if (refresh)\n            pre[j] = wl[j];             /* Alg. 2: pre_weight = w'           */",
                                 "        REAL keep_ = wl[j]; (void)keep_;"),
    "divisor k dropped":        ("((double)lr * (double)k)", "((double)lr)"),
    "1-m dropped":              ("(1.0 - (double)m)", "(1.0)"),
    "pull one step early":      ("if (d % s->k == s->k - 1) {", "if ((d + 1) % s->k == s->k - 1) {"),
    "hand-over one step late":  ("s->num == s->W - 1", "s->num == s->W"),
    "w_loc not broadcast":      ("copy_n(n, s->wl + (size_t)i * n, s->wloc + (size_t)i * n);", ";"),
    "pull before server update": None,   # built by hand below
    "exact w_minus ignored":    ("REAL q = pre_scale * pre[j];", "REAL q = pre[j];"),
    "worker's gradient mixed up": ("NAME(ssd_oracle_glu)(n, s->k, g[i],", "NAME(ssd_oracle_glu)(n, s->k, g[0],"),
}


def mutate(src, name):
    if name == "refresh takes updated w'":
        old, new = MUTATIONS[name]
        assert src.count(old) == 1
        src = src.replace(old, new)
        old2 = "        wl[j] = wl[j] - u6;             /* Eq. (glu-update), descent         */"
        assert src.count(old2) == 1
        return src.replace(old2, old2 + "\n        if (refresh) pre[j] = wl[j];")
    if name == "pull before server update":
        # the pulled weight misses this iteration's server update
        old = "        NAME(ssd_oracle_server)(n, K, g, s->rescale, s->lr, s->m, s->wd,\n                                s->w, s->mom);\n        /* local update with GLU,"
        assert src.count(old) == 1
        src = src.replace(old, "        /* local update with GLU,")
        old2 = "        kind = 2;\n        if (d % s->k == s->k - 1) {\n            for (int i = 0; i < K; ++i)\n                copy_n(n, s->w, s->wl + (size_t)i * n);    /* Pull w_t      */\n            kind = 3;\n        }"
        assert src.count(old2) == 1
        return src.replace(old2, old2 + "\n        NAME(ssd_oracle_server)(n, K, g, s->rescale, s->lr, s->m, s->wd, s->w, s->mom);")
    old, new = MUTATIONS[name]
    assert src.count(old) == 1, (name, src.count(old))
    return src.replace(old, new)


def battery():
    """The pins, each with representative parameters; returns the failures."""
    calls = [
        (pins.test_warmup_is_textbook_momentum_sgd, (0, 0, 6)),
        (pins.test_warmup_is_textbook_momentum_sgd, (4, 12, 12)),
        (pins.test_single_worker_aggregate_is_local_gradient, ()),
        (pins.test_constant_gradient_closed_form, ()),
        (pins.test_server_identity_of_section_3_2_1, ()),
        (pins.test_brute_force_exact_dyadic, ()),
        (pins.test_brute_force_general, ("f64", 3, 4, 3)),
        (pins.test_brute_force_general, ("f32", 4, 1, 0)),
        (pins.test_schedule_matches_hand_trace_of_algorithm_1, ()),
        (pins.test_schedule_matches_algorithm_1_counters, (5, 2)),
        (pins.test_grad_sync_closed_form_and_limit, (2,)),
        (pins.test_glu_reduces_to_local_sgd_of_eq_worker, ()),
        (pins.test_glu_pure_decay, ()),
        (pins.test_boundary_step_matches_server_steady_state, ()),
        (pins.test_pull_and_pre_weight_invariants, ("f64",)),
        (pins.test_first_local_update_has_zero_grad_sync, ()),
        (pins.test_exact_w_minus_follows_identity_of_section_3_2_1, ()),
        (pins.test_exact_w_minus_differs_from_default_only_by_the_decay_term, ()),
    ]
    failed = []
    for f, args in calls:
        try:
            f(*args)
        except AssertionError:
            failed.append(f.__name__)
    return failed


def test_unmutated_oracle_passes_the_battery():
    assert battery() == []


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_catch_planted_mistake(name, tmp_path):
    src = mutate(open(obuild.SRC).read(), name)
    csrc = tmp_path / "mutant.c"
    csrc.write_text(src)
    saved = dict(O._libs)
    try:
        for sfx, real in obuild.VARIANTS.items():
            so = str(tmp_path / ("mutant_%s.so" % sfx))
            subprocess.check_call(["gcc"] + obuild.FLAGS + ["-DREAL=" + real, "-DSFX=" + sfx, str(csrc), "-o", so])
            O._libs[sfx] = ctypes.CDLL(so)
        failed = battery()
    finally:
        O._libs.clear()
        O._libs.update(saved)
    assert failed, "no pin noticed the planted mistake %r" % name
