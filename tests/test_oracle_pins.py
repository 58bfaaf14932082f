"""Pins of the CPU oracle against things other than itself.

Each test names the passage of the SSD-SGD paper (or the mathematical fact)
that fixes the expected value.  None of them needs a GPU.
"""
import os
from fractions import Fraction as Fr

import numpy as np
import pytest
import torch

from oracle.ssd_oracle import (KIND_DELAY, KIND_DELAY_PULL, KIND_WARMUP,
                               KIND_WARMUP_LAST, Oracle)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f32(x):
    return float(np.float32(x))


def rand_grads(rng, K, n, scale=1e-2):
    return [rng.standard_normal(n).astype(np.float32) * np.float32(scale)
            for _ in range(K)]


# ---------------------------------------------------------------------------
# (a) warm-up stage and k = 0 are plain synchronous momentum SGD
#     (Alg. 1 warm-up loop; Sec. 3.4: the server is unchanged from SSGD).
#     Reference: torch.optim.SGD in float64.  PyTorch keeps buf = m*buf + g',
#     w -= lr*buf, which is the rule of Sec. 3.2.1 with mom = -lr*buf.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("k,W,steps", [(0, 0, 12), (0, 5, 12), (4, 12, 12)])
def test_warmup_is_textbook_momentum_sgd(k, W, steps):
    rng = np.random.default_rng(1)
    n, K = 37, 4
    lr, m, wd = f32(0.1), f32(0.9), f32(1e-4)
    w0 = rng.standard_normal(n).astype(np.float32)
    o = Oracle(w0, K=K, k=k, W=W, lr=lr, m=m, wd=wd, mode="f64")
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=lr, momentum=m, weight_decay=wd,
                          dampening=0, nesterov=False)
    for t in range(steps):
        g = rand_grads(rng, K, n)
        kind = o.step(g)
        assert kind in (KIND_WARMUP, KIND_WARMUP_LAST)
        p.grad = torch.tensor(np.mean(np.stack(g).astype(np.float64), axis=0))
        opt.step()
        np.testing.assert_allclose(o.w, p.detach().numpy(), rtol=1e-12,
                                   atol=1e-15)
        buf = opt.state[p]["momentum_buffer"].numpy()
        np.testing.assert_allclose(o.mom, -lr * buf, rtol=1e-12, atol=1e-16)
        # during warm-up every worker computes on the pulled global weight
        for i in range(K):
            assert np.array_equal(o.wloc[i], o.w)


# ---------------------------------------------------------------------------
# (b) K = 1: the aggregated gradient is the local gradient.  K = 2 identical
#     workers: g+g and *0.5 are exact, so the result is bit-identical too.
# ---------------------------------------------------------------------------
def test_single_worker_aggregate_is_local_gradient():
    rng = np.random.default_rng(2)
    n = 101
    w0 = rng.standard_normal(n).astype(np.float32)
    lr, m, wd = 0.1, 0.9, 1e-4
    o1 = Oracle(w0, K=1, k=0, W=0, lr=lr, m=m, wd=wd, mode="f32")
    o2 = Oracle(w0, K=2, k=0, W=0, lr=lr, m=m, wd=wd, mode="f32")
    # independent float32 momentum SGD fed g_0 directly (torch CPU, float32,
    # written with the paper's mom = m*mom - lr*(g + wd*w))
    w = torch.tensor(w0)
    mom = torch.zeros(n)
    for t in range(8):
        g = rand_grads(rng, 1, n)
        o1.step(g)
        o2.step([g[0], g[0]])
        gt = torch.tensor(g[0])
        mom = torch.tensor(f32(m)) * mom - torch.tensor(f32(lr)) * (
            gt + torch.tensor(f32(wd)) * w)
        w = w + mom
        assert np.array_equal(o1.w, o2.w) and np.array_equal(o1.mom, o2.mom)
        assert np.array_equal(o1.w, w.numpy())
        assert np.array_equal(o1.mom, mom.numpy())


# ---------------------------------------------------------------------------
# (c) constant gradient, wd = 0: geometric series (the same series the paper
#     sums to get w_minus = lr*grad_sync*(1-m^(t-1))/(1-m), Sec. 3.2.1).
# ---------------------------------------------------------------------------
def test_constant_gradient_closed_form():
    n, K = 5, 4          # 1/K exact in binary32
    lr, m = f32(0.05), f32(0.9)
    w0 = np.linspace(-1, 1, n).astype(np.float32)
    g = np.array([0.5, -0.25, 1.0, 0.0, 2.0], np.float32)
    o = Oracle(w0, K=K, k=0, W=0, lr=lr, m=m, wd=0.0, mode="f64")
    gd = g.astype(np.float64)
    for t in range(1, 60):
        o.step([g] * K)
        mom = -lr * gd * (1 - m ** t) / (1 - m)
        w = w0 - lr * gd / (1 - m) * (t - m * (1 - m ** t) / (1 - m))
        np.testing.assert_allclose(o.mom, mom, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(o.w, w, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------------------
# identity printed in Sec. 3.2.1:
#   (1 - lr*wd)*w_{t-2} - w_{t-1} = lr*grad_{t-2} - m*mom_{t-3}
# holds for every server step; checked in float64.
# ---------------------------------------------------------------------------
def test_server_identity_of_section_3_2_1():
    rng = np.random.default_rng(3)
    n, K = 64, 4
    lr, m, wd = f32(0.1), f32(0.9), f32(1e-2)
    w0 = rng.standard_normal(n).astype(np.float32)
    o = Oracle(w0, K=K, k=3, W=3, lr=lr, m=m, wd=wd, mode="f64")
    for t in range(12):
        g = rand_grads(rng, K, n, 1.0)
        w_old, mom_old = o.w.copy(), o.mom.copy()
        o.step(g)
        gbar = np.mean(np.stack(g).astype(np.float64), axis=0)
        lhs = (1 - lr * wd) * w_old - o.w
        rhs = lr * gbar - m * mom_old
        np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-14)


# ---------------------------------------------------------------------------
# (d) brute force in exact rational arithmetic, written from Alg. 1 / Alg. 2
#     with the paper's own counters (num, wp, loc_update, num % k == k-1).
# ---------------------------------------------------------------------------
def brute_force(w0, grads_per_iter, K, k, wp, lr, m, wd, lr_loc, alpha, beta,
                wd_loc):
    """Exact (Fraction) simulation of one scalar parameter.
    grads_per_iter[it][i] is worker i's gradient in iteration it.
    Returns per-iteration tuples (w, mom, [w'_i], [pre_i], [w_loc_i])."""
    w, mom = Fr(w0), Fr(0)
    wl = [Fr(w0)] * K
    wloc = [Fr(w0)] * K
    pre = [None] * K
    loc_update = [0] * K
    num = 0
    trace = []
    for g in grads_per_iter:
        g = [Fr(x) for x in g]
        gbar = sum(g) / K
        # server, synchronous, every iteration (Eq. server, Sec. 3.2.1)
        mom = -lr * (gbar + wd * w) + m * mom
        w = w + mom
        if num <= wp:
            wloc = [w] * K
            if num == wp:
                wl = [w] * K
        else:
            for i in range(K):
                if loc_update[i] == 0:
                    pre[i] = wl[i]
                gs = (pre[i] - wl[i]) * (1 - m) / (lr * k)
                if loc_update[i] > 0 and loc_update[i] % k == 0:
                    pre[i] = wl[i]
                wl[i] = wl[i] - lr_loc * (alpha * g[i] + wd_loc * wl[i] + beta * gs)
                loc_update[i] += 1
            wloc = list(wl)
            if num % k == k - 1:
                wl = [w] * K
        num += 1
        trace.append((w, mom, list(wl), list(pre), list(wloc)))
    return trace


def _check_against_brute_force(hp, K, k, wp, steps, g_of, w0s, mode, exact):
    lr, m, wd, lr_loc, alpha, beta, wd_loc = hp
    n = len(w0s)
    o = Oracle(np.array(w0s, np.float32), K=K, k=k, W=wp + 1, lr=lr, m=m,
               wd=wd, lr_loc=lr_loc, alpha=alpha, beta=beta, wd_loc=wd_loc,
               mode=mode)
    hpf = [Fr(f32(x)) for x in hp]
    G = [[[g_of(it, i, j) for j in range(n)] for i in range(K)]
         for it in range(steps)]
    traces = [brute_force(Fr(f32(w0s[j])),
                          [[f32(G[it][i][j]) for i in range(K)] for it in range(steps)],
                          K, k, wp, *hpf) for j in range(n)]
    for it in range(steps):
        o.step([np.array(G[it][i], np.float32) for i in range(K)])
        for j in range(n):
            w, mom, wl, pre, wloc = traces[j][it]
            got = [o.w[j], o.mom[j]] + [o.wl[i][j] for i in range(K)] + \
                  [o.wloc[i][j] for i in range(K)]
            exp = [w, mom] + wl + wloc
            if pre[0] is not None:
                got += [o.pre[i][j] for i in range(K)]
                exp += pre
            for a, b in zip(got, exp):
                if exact:
                    assert Fr(float(a)) == b, (it, j, float(a), float(b))
                else:
                    # 1/K is carried as a binary32 configuration value: exact
                    # for K a power of two, 3e-8 off the true mean otherwise
                    tol = 1e-13 if K & (K - 1) == 0 else 2e-7
                    if mode == "f32":
                        tol = 2e-6
                    assert abs(float(a) - float(b)) <= tol * max(1.0, abs(float(b))), \
                        (it, j, float(a), float(b))


def test_brute_force_exact_dyadic():
    """All hyper-parameters and inputs are small dyadic rationals, so every
    intermediate is exactly representable: the binary64 oracle must equal the
    rational result exactly, and so must the binary32 oracle for as long as
    the values fit 24 bits."""
    hp = (0.5, 0.5, 0.25, 2.0, 2.0, 0.5, 0.25)   # lr m wd lr_loc alpha beta wd_loc
    g_of = lambda it, i, j: ((it * 3 + i * 5 + j * 7) % 9 - 4) / 4.0
    _check_against_brute_force(hp, K=2, k=2, wp=1, steps=7, g_of=g_of,
                               w0s=[1.0, -0.5, 0.75], mode="f64", exact=True)
    _check_against_brute_force(hp, K=2, k=2, wp=1, steps=4, g_of=g_of,
                               w0s=[1.0, -0.5, 0.75], mode="f32", exact=True)
    _check_against_brute_force(hp, K=4, k=4, wp=3, steps=10, g_of=g_of,
                               w0s=[1.0, -0.5, 0.75], mode="f64", exact=True)
    # no warm-up stage at all (W = 0, i.e. wp = -1): the steps-delay loop of
    # Alg. 1 starts at iteration 0 with every w'_i = w_0 and pre_weight = w_0
    _check_against_brute_force(hp, K=2, k=2, wp=-1, steps=6, g_of=g_of,
                               w0s=[1.0, -0.5, 0.75], mode="f64", exact=True)
    _check_against_brute_force(hp, K=2, k=2, wp=-1, steps=4, g_of=g_of,
                               w0s=[1.0, -0.5, 0.75], mode="f32", exact=True)


@pytest.mark.parametrize("mode", ["f64", "f32"])
@pytest.mark.parametrize("K,k,wp", [(2, 2, 1), (3, 4, 3), (4, 1, 0), (5, 5, 4), (3, 3, -1), (2, 1, -1)])
def test_brute_force_general(mode, K, k, wp):
    hp = (0.1, 0.9, 1e-4, 0.4, 2.0, 0.5, 1e-4)
    rng = np.random.default_rng(7)
    tab = rng.standard_normal((3 * k + wp + 3, K, 4)) * 0.3
    g_of = lambda it, i, j: float(tab[it, i, j])
    _check_against_brute_force(hp, K, k, wp, steps=3 * k + wp + 3, g_of=g_of,
                               w0s=[1.0, -0.5, 0.75, 0.01], mode=mode,
                               exact=False)


# ---------------------------------------------------------------------------
# schedule against the hand trace of Algorithm 1 and against its counters
# ---------------------------------------------------------------------------
def test_schedule_matches_hand_trace_of_algorithm_1():
    names = {"warmup": KIND_WARMUP, "warmup_last": KIND_WARMUP_LAST,
             "delay": KIND_DELAY, "delay_pull": KIND_DELAY_PULL}
    exp = []
    for line in open(os.path.join(GOLDEN, "alg1_schedule_wp3_k4.txt")):
        if line.strip() and not line.startswith("#"):
            exp.append(names[line.split()[1]])
    o = Oracle(np.zeros(2, np.float32), K=2, k=4, W=4, lr=0.1, m=0.9, wd=0.0)
    g = [np.zeros(2, np.float32)] * 2
    assert [o.step(g) for _ in exp] == exp


@pytest.mark.parametrize("wp,k", [(0, 1), (1, 2), (5, 2), (2, 3), (9, 5), (7, 8)])
def test_schedule_matches_algorithm_1_counters(wp, k):
    assert (1 + wp) % k == 0
    o = Oracle(np.zeros(1, np.float32), K=1, k=k, W=wp + 1, lr=0.1, m=0.9, wd=0.0)
    g = [np.zeros(1, np.float32)]
    for num in range(wp + 1 + 4 * k):
        kind = o.step(g)
        if num < wp:
            assert kind == KIND_WARMUP
        elif num == wp:
            assert kind == KIND_WARMUP_LAST
        else:
            assert kind == (KIND_DELAY_PULL if num % k == k - 1 else KIND_DELAY)


def test_default_hyperparameters_are_the_papers():
    vals = {}
    pairs = []
    for line in open(os.path.join(GOLDEN, "hyperparameters.txt")):
        t = line.split()
        if not t or t[0] == "#":
            continue
        if t[0] == "lr":
            pairs.append((float(t[1]), float(t[3])))
        else:
            vals[t[0]] = float(t[1])
    for lr, loc in pairs:
        o = Oracle(np.zeros(1, np.float32), K=1, k=1, W=0, lr=lr, m=0.9, wd=0.0)
        assert o.s.alpha == vals["alpha"] and o.s.beta == vals["beta"]
        assert abs(o.s.lr_loc - loc) < 1e-6


# ---------------------------------------------------------------------------
# grad_sync (Sec. 3.3) under a constant gradient: closed form and limit.
# With alpha = 0, wd_loc = 0, beta = 1, lr_loc = 1 the GLU step is
# w' <- w' - grad_sync, which exposes grad_sync.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("k", [1, 2, 4])
def test_grad_sync_closed_form_and_limit(k):
    lr, m = f32(0.1), f32(0.9)
    W = 3
    g = np.array([0.5, -2.0, 0.125], np.float32)
    gd = g.astype(np.float64)
    o = Oracle(np.array([1.0, 2.0, -1.0], np.float32), K=2, k=k, W=W, lr=lr,
               m=m, wd=0.0, lr_loc=1.0, alpha=0.0, beta=1.0, wd_loc=0.0,
               mode="f64")
    for _ in range(W):
        o.step([g, g])
    # d = 0: pre_weight was initialised with w' => grad_sync == +0 exactly
    before = o.wl.copy()
    o.step([g, g])
    assert np.array_equal(o.wloc, before)
    # go to the first boundary d = k; there w' is the weight pulled at d = k-1
    for d in range(1, k):
        o.step([g, g])
    before = o.wl.copy()
    assert np.array_equal(before[0], o.w)
    kind = o.step([g, g])
    gs = before - (o.wloc)            # w_loc holds the GLU result
    # pre = w after W server steps, w' = w after W+k server steps:
    # grad_sync = g * (1/k) * sum_{s=W+1}^{W+k} (1 - m^s)
    exp = gd * np.mean([1 - m ** s for s in range(W + 1, W + k + 1)])
    np.testing.assert_allclose(gs[0], exp, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(gs[1], exp, rtol=1e-12, atol=1e-15)

    # long warm-up: grad_sync -> g (Sec. 3.2.1, the limit m^t -> 0)
    W = 400
    o = Oracle(np.array([1.0, 2.0, -1.0], np.float32), K=2, k=k, W=W, lr=lr,
               m=m, wd=0.0, lr_loc=1.0, alpha=0.0, beta=1.0, wd_loc=0.0,
               mode="f64")
    for _ in range(W + k):
        o.step([g, g])
    before = o.wl.copy()
    o.step([g, g])
    np.testing.assert_allclose(before[0] - o.wloc[0], gd, rtol=1e-10)


# ---------------------------------------------------------------------------
# Eq. (glu-update) special cases
# ---------------------------------------------------------------------------
def test_glu_reduces_to_local_sgd_of_eq_worker():
    """beta = 0, alpha = 1, wd_loc = 0: Eq. (worker), w' -= lr_loc * g_i."""
    rng = np.random.default_rng(11)
    n, K, k = 9, 3, 4
    lr_loc = f32(0.3)
    o = Oracle(rng.standard_normal(n).astype(np.float32), K=K, k=k, W=1,
               lr=0.1, m=0.9, wd=1e-4, lr_loc=lr_loc, alpha=1.0, beta=0.0,
               wd_loc=0.0, mode="f64")
    o.step(rand_grads(rng, K, n))
    for d in range(2 * k):
        g = rand_grads(rng, K, n)
        before = o.wl.copy()
        o.step(g)
        for i in range(K):
            np.testing.assert_allclose(o.wloc[i], before[i] - lr_loc * g[i].astype(np.float64),
                                       rtol=1e-14, atol=1e-16)


def test_glu_pure_decay():
    """alpha = beta = 0: w' <- w' * (1 - lr_loc*wd_loc)."""
    rng = np.random.default_rng(12)
    n, K, k = 9, 2, 3
    lr_loc, wd_loc = f32(0.5), f32(0.125)
    o = Oracle(rng.standard_normal(n).astype(np.float32), K=K, k=k, W=1,
               lr=0.1, m=0.9, wd=0.0, lr_loc=lr_loc, alpha=0.0, beta=0.0,
               wd_loc=wd_loc, mode="f64")
    o.step(rand_grads(rng, K, n))
    for d in range(k):
        before = o.wl.copy()
        o.step(rand_grads(rng, K, n))
        np.testing.assert_allclose(o.wloc, before * (1 - lr_loc * wd_loc), rtol=1e-14)


def test_boundary_step_matches_server_steady_state():
    """m = 0.9, alpha = 2, beta = 0.5, lr_loc = 4*lr (Sec. 4.1), wd = 0,
    constant gradient, long warm-up.  The server's steady-state displacement
    is -lr*g/(1-m) = -10*lr*g.  On a boundary step (d > 0, d % k == 0)
    grad_sync ~ g and the local displacement is -lr_loc*(alpha+beta)*g =
    -10*lr*g as well: the local step follows the server only with the descent
    sign in Eq. (glu-update).  At d = 0, grad_sync = 0 and the step is
    -lr_loc*alpha*g = -8*lr*g; right after a boundary grad_sync = g/k."""
    lr = f32(0.1)
    g = np.array([0.5, -2.0, 0.125], np.float32)
    gd = g.astype(np.float64)
    for k in (2, 4):
        W = 400
        o = Oracle(np.array([1.0, 2.0, -1.0], np.float32), K=2, k=k, W=W,
                   lr=lr, m=0.9, wd=0.0, mode="f64")
        for _ in range(W):
            o.step([g, g])
        b = o.wl.copy(); w_b = o.w.copy()
        o.step([g, g])                                  # d = 0
        np.testing.assert_allclose(o.wloc[0] - b[0], -8 * lr * gd, rtol=1e-6)
        np.testing.assert_allclose(o.w - w_b, -10 * lr * gd, rtol=1e-6)
        for d in range(1, k):
            o.step([g, g])
        b = o.wl.copy(); w_b = o.w.copy()
        o.step([g, g])                                  # d = k: boundary
        np.testing.assert_allclose(o.wloc[0] - b[0], -10 * lr * gd, rtol=1e-6)
        np.testing.assert_allclose(o.w - w_b, -10 * lr * gd, rtol=1e-6)
        if k > 1:
            b2 = o.wl.copy()
            o.step([g, g])                              # d = k+1: gs = g/k
            exp = -4 * lr * (2 * gd + 0.5 * gd / k)
            np.testing.assert_allclose(o.wloc[0] - b2[0], exp, rtol=1e-6)


# ---------------------------------------------------------------------------
# invariants stated in prose
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("mode", ["f32", "f64"])
def test_pull_and_pre_weight_invariants(mode):
    rng = np.random.default_rng(21)
    n, K, k, W = 33, 4, 3, 2
    o = Oracle(rng.standard_normal(n).astype(np.float32), K=K, k=k, W=W,
               lr=0.1, m=0.9, wd=1e-4, mode=mode)
    last_pulled = None
    for it in range(W + 4 * k):
        g = rand_grads(rng, K, n)
        pre_wl = o.wl.copy()
        kind = o.step(g)
        if kind == KIND_WARMUP_LAST:
            last_pulled = o.w.copy()
            for i in range(K):
                assert np.array_equal(o.wl[i], o.w)       # w'_{t,i} = w_t
        if kind in (KIND_DELAY, KIND_DELAY_PULL):
            d = o.d - 1
            # Sec. 3.3: all workers hold the same pre_weight ...
            for i in range(1, K):
                assert np.array_equal(o.pre[i], o.pre[0])
            # ... which is the global weight of the previous retrieval
            if d > 0 and d % k == 0:
                assert np.array_equal(o.pre[0], pre_wl[0])
                assert np.array_equal(o.pre[0], last_pulled_prev)
            if kind == KIND_DELAY:
                assert np.array_equal(o.wloc, o.wl)
            else:
                for i in range(K):
                    assert np.array_equal(o.wl[i], o.w)   # Pull: w' = w_t
                assert not np.array_equal(o.wloc[0], o.wl[0])
                last_pulled_prev = o.w.copy()
        if kind == KIND_WARMUP_LAST:
            last_pulled_prev = last_pulled


def test_first_local_update_has_zero_grad_sync():
    """pre_weight is initialised with w' (Alg. 2): the first local update is
    SGD with step lr_loc*alpha on g plus decay, for any beta."""
    rng = np.random.default_rng(5)
    n, K = 17, 2
    w0 = rng.standard_normal(n).astype(np.float32)
    res = []
    for beta in (0.5, 123.0):
        o = Oracle(w0, K=K, k=4, W=1, lr=0.1, m=0.9, wd=1e-4, beta=beta, mode="f32")
        r = np.random.default_rng(6)
        o.step(rand_grads(r, K, n))
        o.step(rand_grads(r, K, n))
        res.append(o.wl.copy())
    assert np.array_equal(res[0], res[1])


# ---------------------------------------------------------------------------
# metamorphic: the rules are jointly linear-homogeneous in (w_0, g)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("p", [-7, 5])
def test_power_of_two_scaling_is_exact_in_binary32(p):
    rng = np.random.default_rng(31)
    n, K, k, W = 50, 3, 2, 2
    w0 = rng.standard_normal(n).astype(np.float32)
    s = np.float32(2.0 ** p)
    a = Oracle(w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    b = Oracle(w0 * s, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    for it in range(W + 3 * k):
        g = rand_grads(rng, K, n)
        a.step(g)
        b.step([x * s for x in g])
        for name in ("w", "mom", "wl", "wloc"):
            assert np.array_equal(getattr(a, name) * s, getattr(b, name)), name


def test_worker_permutation():
    rng = np.random.default_rng(41)
    n, K, k, W = 20, 4, 2, 1
    w0 = rng.standard_normal(n).astype(np.float32)
    perm = [2, 0, 3, 1]
    a = Oracle(w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f64")
    b = Oracle(w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f64")
    for it in range(W + 3 * k):
        g = rand_grads(rng, K, n)
        a.step(g)
        b.step([g[j] for j in perm])
        np.testing.assert_allclose(a.w, b.w, rtol=1e-13, atol=1e-16)
        for i, j in enumerate(perm):
            np.testing.assert_allclose(b.wloc[i], a.wloc[j], rtol=1e-12, atol=1e-15)


def test_binary32_oracle_tracks_binary64_oracle():
    """The two builds of the one source differ by rounding only."""
    rng = np.random.default_rng(51)
    n, K, k, W = 1000, 4, 4, 2
    w0 = rng.standard_normal(n).astype(np.float32)
    a = Oracle(w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    b = Oracle(w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f64")
    for it in range(W + 5 * k):
        g = rand_grads(rng, K, n)
        a.step(g); b.step(g)
    for name in ("w", "mom", "wl", "wloc", "pre"):
        x, y = getattr(a, name).astype(np.float64), getattr(b, name)
        assert np.max(np.abs(x - y)) <= 1e-5 * np.max(np.abs(y)), name


def test_piecewise_calls_equal_step():
    """server + K glu + pull, called one by one, give the state of step()."""
    rng = np.random.default_rng(61)
    n, K, k, W = 40, 3, 2, 1
    w0 = rng.standard_normal(n).astype(np.float32)
    a = Oracle(w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    b = Oracle(w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    g = rand_grads(rng, K, n)
    a.step(g)
    b.server(g)
    for i in range(K):
        b.pull(i)
    for d in range(3 * k):
        g = rand_grads(rng, K, n)
        a.step(g)
        b.server(g)
        for i in range(K):
            b.glu(i, g[i])
        if d % k == k - 1:
            for i in range(K):
                b.pull(i)
            for name in ("w", "mom", "wl", "pre", "wloc"):
                assert np.array_equal(getattr(a, name), getattr(b, name)), name
        else:
            for name in ("w", "mom", "wl", "pre"):
                assert np.array_equal(getattr(a, name), getattr(b, name)), name


# ---------------------------------------------------------------------------
# variant: grad_sync from the exact w_minus of Sec. 3.2.1
# ---------------------------------------------------------------------------
def test_exact_w_minus_follows_identity_of_section_3_2_1():
    """k = 1: at every local update after the first, pre_weight is w_{j-1} and
    w' is w_j (pulled one iteration earlier), so by the identity of Sec. 3.2.1
      (1 - lr*wd)*w_{j-1} - w_j = lr*grad_{j-1} - m*mom_{j-2}
    the exact grad_sync equals (lr*grad - m*mom_prev)*(1-m)/lr, a quantity of
    the server alone.  alpha = 0, wd_loc = 0, beta = 1, lr_loc = 1 expose it:
    w_loc = w' - grad_sync."""
    rng = np.random.default_rng(71)
    n, K, W = 11, 2, 3
    lr, m, wd = f32(0.1), f32(0.9), f32(0.05)
    o = Oracle(rng.standard_normal(n).astype(np.float32), K=K, k=1, W=W, lr=lr, m=m, wd=wd,
               lr_loc=1.0, alpha=0.0, beta=1.0, wd_loc=0.0, exact_w_minus=True, mode="f64")
    prev = None      # (averaged gradient, momentum before the step) of the previous iteration
    for it in range(W + 6):
        g = rand_grads(rng, K, n, 1.0)
        gbar = np.mean(np.stack(g).astype(np.float64), axis=0)
        mom_before = o.mom.copy()
        wl_before = o.wl.copy()
        o.step(g)
        if it > W:   # d >= 1
            gbar_prev, mom_prev = prev
            exp = (lr * gbar_prev - m * mom_prev) * (1 - m) / lr
            np.testing.assert_allclose(wl_before[0] - o.wloc[0], exp, rtol=1e-9, atol=1e-12)
        prev = (gbar, mom_before)


def test_exact_w_minus_differs_from_default_only_by_the_decay_term():
    """With wd = 0 the two forms coincide bit for bit; with wd > 0 they differ."""
    rng = np.random.default_rng(72)
    n, K, k, W = 30, 2, 2, 2
    w0 = rng.standard_normal(n).astype(np.float32)
    gs = [rand_grads(rng, K, n) for _ in range(W + 5)]
    for wd, same in ((0.0, True), (1e-2, False)):
        a = Oracle(w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=wd, wd_loc=0.0, mode="f32")
        b = Oracle(w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=wd, wd_loc=0.0, exact_w_minus=True, mode="f32")
        for g in gs:
            a.step(g); b.step(g)
        assert np.array_equal(a.w, b.w)                       # the server never depends on it
        assert np.array_equal(a.wl, b.wl) == same
