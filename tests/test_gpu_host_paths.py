"""GPU tests of the host-side paths of the library that the plain parity
tests do not reach: eviction in the device-resident cache of gradient-pointer
tables (also across streams), and every refusal (SSD_ESTATE / SSD_EALIGN) --
each followed by valid calls whose state must still equal the oracle's bit
for bit, i.e. a failing call leaves the state untouched.  Every kernel that
runs here is a normal launch; a refusal happens on the host before anything
is enqueued."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle.ssd_oracle import Oracle
from paper_2012_05396_amd import binding as B
from ssd_harness import Model, compare_state, run_schedule

pytestmark = pytest.mark.gpu

SIZES = [3000, 257, 64, 5]


def test_fused_table_cache_evicts_every_step():
    """Eleven distinct gradient sets cycled through ssd_step: the cache holds
    eight tables, so from the ninth iteration on every call evicts the least
    recently used one and uploads anew (Alg. 1: only the gradient pointers
    change from iteration to iteration)."""
    print("case: 11 gradient sets, 8 cache slots", flush=True)
    run_schedule(SIZES, K=3, k=3, W=2, steps=2 + 31, P=11, seed=21)


def test_table_evicted_from_another_stream():
    """Tables first used on stream A are evicted by calls on stream B while A's
    launches may still be in flight: the library must wait for A before it
    overwrites a table A's kernels read.  Bursts of iterations alternate
    between the streams without a device-wide wait in between; the caller
    orders the streams' data dependencies with events, as ssd.h asks."""
    print("case: eviction across streams", flush=True)
    K, k, W, P = 2, 2, 1, 10
    m = Model(SIZES, K, P=P, seed=33)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    cfg = B.make_config(SIZES, K, k, W, 0.1, 0.9, 1e-4, stream=sa.cuda_stream)
    torch.cuda.synchronize()
    ctx = B.Context(cfg, m.weights)
    o = Oracle(m.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    tables = [B.GradTable(g) for g in m.g_dev]
    it = 0
    cur, other = sa, sb
    for burst in range(8):
        n = 8 if burst == 0 else 5       # first burst fills all eight slots from stream A
        for _ in range(n):
            ctx.ssd_step(tables[it % P])
            o.step(m.g_host[it % P])
            it += 1
        ev = torch.cuda.Event()
        ev.record(cur)
        other.wait_event(ev)             # the next burst reads what this one wrote
        cur, other = other, cur
        ctx.ssd_set_stream(cur)
        if burst % 2 == 1:
            compare_state(ctx, m, o, exact=True, where="two-stream eviction, burst %d" % burst)
    compare_state(ctx, m, o, exact=True, where="two-stream eviction, end")
    ctx.close()


def _raw_table(grads):
    """[K][T] pointer table as ssd_step takes it, plus the rows to edit."""
    rows = [(C.c_void_p * len(r))(*[t.data_ptr() for t in r]) for r in grads]
    table = (C.c_void_p * len(rows))(*[C.cast(r, C.c_void_p).value for r in rows])
    return table, rows


def _refused(rc, ctx, code):
    msg = B.lib.ssd_last_error(ctx.h).decode()
    assert rc == code, (rc, code, msg)
    assert len(msg) > 10
    return msg


def test_refusals_leave_the_state_untouched():
    """Each SSD_ESTATE / SSD_EALIGN refusal of the piecewise calls and of
    ssd_step, provoked inside a valid piecewise schedule that goes on
    afterwards and must match the oracle at every iteration."""
    print("case: refusals", flush=True)
    K, k, W, P = 2, 2, 1, 3
    m = Model(SIZES, K, P=P, seed=44)
    cfg = B.make_config(SIZES, K, k, W, 0.1, 0.9, 1e-4, stream=torch.cuda.current_stream().cuda_stream)
    ctx = B.Context(cfg, m.weights)
    o = Oracle(m.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    g = m.g_dev
    row = lambda p, i: (C.c_void_p * len(SIZES))(*[t.data_ptr() for t in g[p][i]])
    glu = lambda p, i: B.lib.ssd_worker_glu_update(ctx.h, i, row(p, i))

    def step(p):
        table, rows = _raw_table(g[p])      # `rows` must outlive the call: the table points into them
        return B.lib.ssd_step(ctx.h, table)

    # iteration 0 = last warm-up iteration.  Before it: no worker has local weights.
    assert "no local weights" in _refused(glu(0, 0), ctx, B.SSD_ESTATE)
    # a gradient pointer that is not aligned to its element size
    table, rows = _raw_table(g[0])
    rows[1][2] = rows[1][2] + 2
    assert "aligned" in _refused(B.lib.ssd_step(ctx.h, table), ctx, B.SSD_EALIGN)
    bad_row = row(0, 0)
    bad_row[0] = bad_row[0] + 1
    assert step(0) == B.SSD_OK
    o.step(m.g_host[0])
    compare_state(ctx, m, o, where="after warm-up")
    _refused(B.lib.ssd_worker_glu_update(ctx.h, 0, bad_row), ctx, B.SSD_EALIGN)
    _refused(B.lib.ssd_worker_glu_update(ctx.h, K, row(0, 0)), ctx, B.SSD_EINVAL)

    # iteration 1: d = 0, pre_weight initialised; piecewise
    ctx.ssd_server_aggregate_update(g[1])
    assert glu(1, 0) == B.SSD_OK
    assert "different local update counts" in _refused(step(1), ctx, B.SSD_ESTATE)  # half of an init round done
    assert "slowest" in _refused(glu(1, 0), ctx, B.SSD_ESTATE)          # worker 0 would run ahead
    assert glu(1, 1) == B.SSD_OK
    o.step(m.g_host[1])
    compare_state(ctx, m, o, where="after d=0")

    # iteration 2: d = 1, then the Pull
    ctx.ssd_server_aggregate_update(g[2])
    assert glu(2, 0) == B.SSD_OK
    assert "different local update counts" in _refused(step(2), ctx, B.SSD_ESTATE)
    assert glu(2, 1) == B.SSD_OK
    # d = 2 would refresh pre_weight from w': refused until the worker has pulled
    assert "must pull" in _refused(glu(0, 0), ctx, B.SSD_ESTATE)
    assert "pulled" in _refused(step(0), ctx, B.SSD_ESTATE)
    ctx.ssd_worker_pull(0)
    assert "pulled" in _refused(step(0), ctx, B.SSD_ESTATE)             # worker 1 has not yet
    ctx.ssd_worker_pull(1)
    o.step(m.g_host[2])
    compare_state(ctx, m, o, where="after d=1 and the Pull")

    # iterations 3, 4: fused again, from the arrays the piecewise calls left
    for it in (3, 4):
        assert step(it % P) == B.SSD_OK
        o.step(m.g_host[it % P])
        compare_state(ctx, m, o, where="fused after piecewise, it=%d" % it)

    # d = 4 is a refresh.  Workers that pulled different global weights cannot
    # share one pre_weight: worker 0 pulls, the servers move on, worker 1 pulls.
    ctx.ssd_materialize()
    ctx.ssd_worker_pull(0)
    ctx.ssd_server_aggregate_update(g[0])
    ctx.ssd_worker_pull(1)
    assert "pulled" in _refused(step(1), ctx, B.SSD_ESTATE)
    assert glu(1, 0) == B.SSD_OK
    assert "another global weight" in _refused(glu(1, 1), ctx, B.SSD_ESTATE)
    torch.cuda.synchronize()
    ctx.close()


def test_refusals_without_a_delay_stage():
    print("case: refusals, k = 0", flush=True)
    m = Model(SIZES, 2, P=1, seed=45)
    ctx = B.Context(B.make_config(SIZES, 2, 0, 0, 0.1, 0.9, 1e-4,
                                  stream=torch.cuda.current_stream().cuda_stream), m.weights)
    r = (C.c_void_p * len(SIZES))(*[t.data_ptr() for t in m.g_dev[0][0]])
    assert "delay_k = 0" in _refused(B.lib.ssd_worker_glu_update(ctx.h, 0, r), ctx, B.SSD_ESTATE)
    assert "delay_k = 0" in _refused(B.lib.ssd_worker_pull(ctx.h, 0), ctx, B.SSD_ESTATE)
    o = Oracle(m.w0, K=2, k=0, W=0, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    ctx.ssd_step(m.g_dev[0])
    o.step(m.g_host[0])
    compare_state(ctx, m, o, where="k = 0 after refusals")
    ctx.close()


def test_cache_policy_choice_and_override():
    """Auto: ordinary accesses (and no occupancy cap) while everything one
    iteration touches fits the 256 MiB last-level cache, else non-temporal ones;
    either can be forced.  Bits never depend on it (every schedule test runs
    both policies side by side); here: what the state view reports."""
    print("case: cache policy", flush=True)
    numel = [300000, 70000]          # 370 K elements: 35 arrays at K = 16 are 52 MB
    w = [torch.zeros(n, device="cuda") for n in numel]
    stream = torch.cuda.current_stream().cuda_stream
    for policy, expect in ((B.SSD_CACHE_AUTO, 0), (B.SSD_CACHE_STREAMING, 1), (B.SSD_CACHE_RESIDENT, 0)):
        ctx = B.Context(B.make_config(numel, 16, 2, 1, 0.1, 0.9, 1e-4, stream=stream, cache_policy=policy), w)
        assert ctx.ssd_get_state().streaming == expect
        ctx.close()
    # 8 Mi elements: K = 1 touches 5 arrays = 160 MiB -> resident; K = 4 touches 11 = 352 MiB -> streaming
    big = [torch.zeros(8 << 20, device="cuda")]
    for K, expect in ((1, 0), (4, 1)):
        ctx = B.Context(B.make_config([8 << 20], K, 2, 1, 0.1, 0.9, 1e-4, stream=stream), big)
        assert ctx.ssd_get_state().streaming == expect
        ctx.close()
    # 16-bit gradients count half: K = 3 with bfloat16 touches 3*2 + 6*4 = 30 B per element = 240 MiB -> resident,
    # with binary32 gradients 36 B = 288 MiB -> streaming
    for gd, expect in ((B.SSD_GRAD_BF16, 0), (B.SSD_GRAD_F32, 1)):
        ctx = B.Context(B.make_config([8 << 20], 3, 2, 1, 0.1, 0.9, 1e-4, stream=stream, grad_dtype=gd), big)
        assert ctx.ssd_get_state().streaming == expect
        ctx.close()


def test_two_contexts_on_two_host_threads():
    """A context belongs to one host thread at a time; different contexts may
    be driven from different threads at once (ctypes releases the GIL during
    the calls).  Each thread has its own stream, weights, gradients and oracle;
    both use a 2-wave occupancy cap, whose LDS slice above 64 KiB makes the
    launcher raise the kernel's dynamic-LDS limit once per device -- the one
    piece of state that contexts share."""
    import threading
    print("case: two host threads", flush=True)
    K, k, W, steps = 3, 2, 1, 12
    errors = []

    def work(seed):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                m = Model(SIZES, K, seed=seed)
                ctx = B.Context(B.make_config(SIZES, K, k, W, 0.1, 0.9, 1e-4, stream=stream.cuda_stream,
                                              waves_per_cu=2, cache_policy=B.SSD_CACHE_STREAMING), m.weights)
                o = Oracle(m.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
                tables = [B.GradTable(g) for g in m.g_dev]
                for it in range(steps):
                    ctx.ssd_step(tables[it % 3])
                    o.step(m.g_host[it % 3])
                stream.synchronize()
                compare_state(ctx, m, o, exact=True, where="thread %d" % seed)
                ctx.close()
        except BaseException as e:      # reported by the main thread
            errors.append(e)

    threads = [threading.Thread(target=work, args=(s,)) for s in (71, 72)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
