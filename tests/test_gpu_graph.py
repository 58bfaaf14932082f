"""ssd_step under HIP graph capture: one k-cycle of the steps-delay stage is
captured once and replayed; every replay must leave the state the oracle has
after the same number of iterations.

What makes this legal: in steady state ssd_step enqueues exactly one kernel
launch -- its pointer tables are resident after the first use of a gradient set
(the library keeps 8 of them), it allocates nothing and clears nothing -- and a
whole k-cycle starting at a cycle boundary returns the context's recorded flags
to their values at the start, so the launches of the next cycle are the same.
Replays do not advance the context's iteration counters."""
import numpy as np
import pytest
import torch

from ssd_harness import Model, compare_state

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("K,k,numel", [(4, 4, [5000, 17, 1025, 64]), (3, 2, [300, 4097])])
def test_replayed_cycle_matches_the_oracle(K, k, numel):
    print("case: graph replay K=%d k=%d" % (K, k), flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    W, P = 1, k                      # one gradient set per iteration of the cycle
    model = Model(numel, K, P=P, seed=5 + K)
    side = torch.cuda.Stream()
    cfg = B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, stream=side.cuda_stream)
    ctx = B.Context(cfg, model.weights)
    o = Oracle(model.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    tables = [B.GradTable(g) for g in model.g_dev]
    torch.cuda.synchronize()

    def eager(n):
        # iteration W + j uses gradient set j % k, also inside the graph
        for _ in range(n):
            j = (ctx.ssd_get_state().iterations - W) % P
            ctx.ssd_step(tables[j])
            o.step(model.g_host[j])

    # warm-up iteration, then two whole cycles eagerly on the side stream:
    # every table is resident, the next iteration starts a cycle (d % k == 0)
    with torch.cuda.stream(side):
        ctx.ssd_step(tables[0]); o.step(model.g_host[0])      # the SSGD iteration (index 0 < W)
        eager(2 * k)
    side.synchronize()
    compare_state(ctx, model, o, exact=True, where="before capture")
    assert ctx.ssd_get_state().local_updates % k == 0

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side, capture_error_mode="thread_local"):
        for j in range(k):
            ctx.ssd_step(tables[j])
    # capture ran nothing: the state is still the oracle's
    compare_state_before = [w.clone() for w in model.weights]
    torch.cuda.synchronize()
    for a, b in zip(compare_state_before, model.weights):
        assert torch.equal(a, b)

    junk = torch.zeros(1 << 20, device="cuda")
    for rep in range(4):
        graph.replay()
        for j in range(k):
            o.step(model.g_host[j])
        torch.cuda.synchronize()
        compare_state(ctx, model, o, exact=True, where="replay %d" % rep)
        # the program's own eager work and synchronisations between replays
        junk.add_(1.0).mul_(0.5)
        _ = float(junk.sum())
        torch.cuda.synchronize()
    # eager steps continue correctly after the replays (flags are periodic)
    with torch.cuda.stream(side):
        for j in range(k + 1):
            ctx.ssd_step(tables[j % P]); o.step(model.g_host[j % P])
    torch.cuda.synchronize()
    compare_state(ctx, model, o, exact=True, where="eager after replays")
    ctx.close()


def test_capture_on_a_stream_other_than_the_upload_stream():
    """Tables uploaded on the stream given at init, capture on a second stream
    after ssd_set_stream: the first eager use on the new stream takes the one
    cross-stream wait, the captured calls are bare launches."""
    print("case: graph replay after ssd_set_stream", flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    numel, K, k, W = [3000, 5, 1024], 2, 3, 0
    model = Model(numel, K, P=k, seed=31)
    main = torch.cuda.current_stream()
    ctx = B.Context(B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, stream=main.cuda_stream), model.weights)
    o = Oracle(model.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    tables = [B.GradTable(g) for g in model.g_dev]
    for j in range(k):
        ctx.ssd_step(tables[j]); o.step(model.g_host[j])
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    ctx.ssd_set_stream(side)
    with torch.cuda.stream(side):
        for j in range(k):
            ctx.ssd_step(tables[j]); o.step(model.g_host[j])
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side, capture_error_mode="thread_local"):
        for j in range(k):
            ctx.ssd_step(tables[j])
    for rep in range(3):
        graph.replay()
        for j in range(k):
            o.step(model.g_host[j])
        torch.cuda.synchronize()
        compare_state(ctx, model, o, exact=True, where="set_stream replay %d" % rep)
        _ = float(torch.ones(1000, device="cuda").sum())
    ctx.close()
