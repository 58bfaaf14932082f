"""GPU parity: the HIP library against the CPU oracle, through the C ABI.

Bit-exact against the binary32 oracle (same rounding sequence), and within
1e-5 (per tensor, max |a-b| / max |b|) against the binary64 oracle."""
import numpy as np
import pytest
import torch

from ssd_harness import (Model, bits, cat, compare_state, effective_w_loc, effective_w_local,
                         run_schedule)

pytestmark = pytest.mark.gpu

ODD = [1, 3, 4, 5, 63, 64, 65, 1023, 1024, 1025, 4097, 2051]


@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 8, 16])
def test_tiny_odd_tensors_bit_exact(K):
    print("case: odd tensors K=%d" % K, flush=True)
    run_schedule(ODD, K=K, k=3, W=2, steps=2 + 7, seed=K)


@pytest.mark.parametrize("k,W", [(0, 0), (0, 3), (1, 0), (1, 2), (2, 0), (2, 1), (4, 2), (5, 3)])
def test_schedules_bit_exact(k, W):
    print("case: schedule k=%d W=%d" % (k, W), flush=True)
    run_schedule(ODD, K=4, k=k, W=W, steps=W + 3 * max(k, 1) + 1, seed=10 * k + W)


@pytest.mark.parametrize("w_shift,g_shift", [(1, 0), (0, 1), (3, 2)])
def test_misaligned_pointers_take_scalar_path(w_shift, g_shift):
    print("case: misaligned w_shift=%d g_shift=%d" % (w_shift, g_shift), flush=True)
    run_schedule(ODD, K=3, k=2, W=1, steps=6, w_shift=w_shift, g_shift=g_shift, seed=5)


@pytest.mark.parametrize("K,w_shift,g_shift", [(9, 0, 1), (11, 1, 2), (16, 3, 0), (16, 0, 0)])
def test_more_than_8_workers_on_the_scalar_path_and_large_chunks(K, w_shift, g_shift):
    """K > 8: the local weights are interleaved by block.  Misaligned caller
    pointers send every lane element by element; chunks of several tiles make
    the interleaved unit larger than a tile; the exact-w_minus variant is its
    own kernel."""
    print("case: more than 8 workers K=%d w_shift=%d g_shift=%d" % (K, w_shift, g_shift), flush=True)
    run_schedule(ODD, K=K, k=3, W=1, steps=1 + 7, w_shift=w_shift, g_shift=g_shift, seed=100 + K)
    run_schedule([20000, 8193, 7], K=K, k=2, W=0, steps=5, chunk_elems=1024, w_shift=w_shift, g_shift=g_shift,
                 seed=200 + K, hp=dict(lr=0.1, momentum=0.9, wd=1e-4, grad_sync_exact=1))


BIG = [9000, 8192 + 3, 64, 10001, 20000, 12345, 8192, 5]   # tensors of 32 tiles and more get a lead-in


@pytest.mark.parametrize("K,w_shift,g_shift,chunk", [(3, 0, 0, 0), (4, 0, 4, 0), (2, 0, 1, 0), (3, 4, 0, 1024),
                                                    (9, 0, 0, 0), (16, 8, 8, 0), (5, 1, 0, 0), (8, 0, 0, 512)])
def test_lead_in_of_large_tensors(K, w_shift, g_shift, chunk):
    """Tensors of at least 32 tiles start inside their first arena block so that
    tiles follow the 1 KiB grid of the weight pointer (the harness places tensors
    at multiples of 256 bytes plus the shift, so all four phases occur).  The
    gradient buffers share the phase (shift equal), have another one (still
    16-byte aligned: 128-bit path) or are not 16-byte aligned (element by
    element, with the lead-in of the aligned weights); misaligned weights get
    no lead-in.  Fused step, also against the piecewise calls."""
    print("case: lead-in K=%d w_shift=%d g_shift=%d chunk=%d" % (K, w_shift, g_shift, chunk), flush=True)
    from paper_2012_05396_amd import binding as B
    model, _ = run_schedule(BIG, K=K, k=2, W=1, steps=6, w_shift=w_shift, g_shift=g_shift, chunk_elems=chunk,
                            seed=300 + K)
    # the state view reports where each tensor starts; large aligned tensors do not start on a block boundary
    cfg = B.make_config(BIG, K, 2, 1, 0.1, 0.9, 1e-4, stream=torch.cuda.current_stream().cuda_stream,
                        chunk_elems=chunk)
    ctx = B.Context(cfg, model.weights)
    v = ctx.ssd_get_state()
    C = v.chunk_elems
    for t, n in enumerate(BIG):
        a = model.weights[t].data_ptr()
        lead = (a % 1024) // 4 if (n >= 32 * 256 and a % 16 == 0) else 0
        assert v.tensor_offset[t] % C == lead, (t, v.tensor_offset[t], lead)
    # the host-only planner names the same layout from the pointer values alone
    off, blocks, nbytes = B.ssd_plan_arena(cfg, [w.data_ptr() for w in model.weights])
    assert off == [v.tensor_offset[t] for t in range(len(BIG))] and len(blocks) == v.num_chunks
    assert nbytes <= B.ssd_workspace_bytes(cfg)
    ctx.close()


@pytest.mark.parametrize("K", [3, 11])
def test_lead_in_piecewise_equals_fused(K):
    """Piecewise calls on tensors with lead-ins; K = 11: the GLU and Pull kernels
    walk the interleaved local weights with their block stride."""
    print("case: lead-in, piecewise K=%d" % K, flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    k, W = 2, 1
    m = Model(BIG, K, seed=55)
    ctx = B.Context(B.make_config(BIG, K, k, W, 0.1, 0.9, 1e-4, stream=torch.cuda.current_stream().cuda_stream),
                    m.weights)
    o = Oracle(m.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    for it in range(W + 2 * k + 1):
        p = it % 3
        ctx.ssd_server_aggregate_update(m.g_dev[p])
        if it == W - 1:
            for i in range(K):
                ctx.ssd_worker_pull(i)
        elif it >= W:
            for i in range(K):
                ctx.ssd_worker_glu_update(i, m.g_dev[p][i])
            if (it - W) % k == k - 1:
                for i in range(K):
                    ctx.ssd_worker_pull(i)
        o.step(m.g_host[p])
        compare_state(ctx, m, o, exact=True, where="lead-in piecewise it=%d" % it)
    ctx.close()


def test_many_tiny_tensors():
    """2000 tensors of 1 .. 300 elements with K = 16 workers: one block and one
    table record per tensor, 38 000 pointers per gradient set."""
    print("case: many tiny tensors", flush=True)
    rng = np.random.default_rng(5)
    sizes = [int(x) for x in rng.integers(1, 301, size=2000)]
    run_schedule(sizes, K=16, k=2, W=1, steps=6, seed=6, P=2, check_every=3)
    run_schedule(sizes[:500], K=3, k=4, W=2, steps=8, seed=7, P=2, check_every=4)


@pytest.mark.parametrize("K", [6, 7, 9, 10, 11, 12, 13, 14, 15])
def test_remaining_worker_counts(K):
    print("case: K=%d" % K, flush=True)
    run_schedule([5000, 17], K=K, k=2, W=1, steps=5, seed=K)


def test_hyperparameters_and_lr_change():
    print("case: hyper-parameters", flush=True)
    hp = dict(lr=0.05, momentum=0.8, wd=1e-3, lr_loc=0.3, alpha=1.5, beta=0.25, wd_loc=2e-3,
              rescale_grad=0.125)
    run_schedule(ODD, K=4, k=2, W=2, steps=9, hp=hp, seed=3,
                 lr_changes={4: (0.02, 0.1), 7: (0.2, 0.8)})


def test_large_chunks_and_multi_pass():
    print("case: chunk sizes", flush=True)
    for ce in (256, 1024, 2048, 8192, 0):
        run_schedule([20000, 8192, 8193, 7], K=4, k=2, W=1, steps=5, chunk_elems=ce, seed=ce)


def test_plain_oracle_within_tolerance():
    print("case: plain oracle", flush=True)
    run_schedule([30000, 513, 64], K=8, k=4, W=2, steps=2 + 20, mode="f64", check_every=22, seed=9)


def test_special_values_propagate():
    """NaN / Inf / denormals / signed zero follow IEEE rules on both sides."""
    print("case: special values", flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    numel = [64, 5]
    K, k, W = 2, 2, 1
    model = Model(numel, K, P=2, seed=1)
    special = np.array([np.nan, np.inf, -np.inf, 1e-45, -1e-45, 1e-39, 0.0, -0.0, 3e38, -3e38,
                        1e-38, 1.17549435e-38], np.float32)
    for p in range(2):
        for i in range(K):
            h = model.g_host[p][i]
            h[:special.size] = np.roll(special, p + i)
            model._scatter(model.g_dev[p][i], h)
    model.w0[20:20 + special.size] = special
    model._scatter(model.weights, model.w0)
    cfg = B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, device=0,
                        stream=torch.cuda.current_stream().cuda_stream)
    ctx = B.Context(cfg, model.weights)
    o = Oracle(model.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    with np.errstate(all="ignore"):
        for it in range(6):
            ctx.ssd_step(model.g_dev[it % 2])
            o.step(model.g_host[it % 2])
            compare_state(ctx, model, o, exact=True, where="special it=%d" % it)
    ctx.close()


def test_piecewise_calls_equal_fused_step():
    """server + K x glu (+ K x pull) == ssd_step, bit for bit (and == oracle)."""
    print("case: piecewise", flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    numel, K, k, W = ODD, 4, 3, 2
    ma = Model(numel, K, seed=77)
    mb = Model(numel, K, seed=77)
    s = torch.cuda.current_stream().cuda_stream
    ca = B.Context(B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, stream=s, chunk_elems=256), ma.weights)
    cb = B.Context(B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, stream=s, chunk_elems=256), mb.weights)
    o = Oracle(ma.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    for it in range(W + 3 * k + 2):
        p = it % 3
        ca.ssd_step(ma.g_dev[p])
        o.step(ma.g_host[p])
        cb.ssd_server_aggregate_update(mb.g_dev[p])
        if it == W - 1:
            for i in range(K):
                cb.ssd_worker_pull(i)
        elif it >= W:
            d = it - W
            order = list(range(K)) if d % 2 == 0 else list(reversed(range(K)))
            for i in order:
                cb.ssd_worker_glu_update(i, mb.g_dev[p][i])
            if d % k == k - 1:
                for i in range(K):
                    cb.ssd_worker_pull(i)
        torch.cuda.synchronize()
        assert np.array_equal(bits(cat(ma.weights)), bits(cat(mb.weights)))
        names = ["mom"] + (["pre"] if it >= W else [])
        for nm in names:
            assert np.array_equal(bits(cat(ca.state_tensors(nm))), bits(cat(cb.state_tensors(nm)))), (it, nm)
        if it >= W - 1:
            for i in range(K):
                assert np.array_equal(bits(effective_w_local(ca, ma, i)),
                                      bits(effective_w_local(cb, mb, i))), (it, i)
                assert np.array_equal(bits(effective_w_loc(ca, ma, i)),
                                      bits(effective_w_loc(cb, mb, i))), (it, i)
        compare_state(cb, mb, o, exact=True, where="piecewise it=%d" % it)
    ca.close(); cb.close()


def test_homogeneity_power_of_two_scaling():
    """Scaling w_0 and all gradients by 2^p scales every output by 2^p."""
    print("case: homogeneity", flush=True)
    from paper_2012_05396_amd import binding as B
    numel, K, k, W = [3000, 77], 4, 2, 1
    res = []
    for scale in (1.0, 2.0 ** -6):
        m = Model(numel, K, seed=4)
        for w in m.weights:
            w.mul_(scale)
        for p in m.g_dev:
            for row in p:
                for g in row:
                    g.mul_(scale)
        ctx = B.Context(B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4,
                                      stream=torch.cuda.current_stream().cuda_stream), m.weights)
        for it in range(W + 2 * k + 1):
            ctx.ssd_step(m.g_dev[it % 3])
        ctx.ssd_materialize()
        torch.cuda.synchronize()
        res.append([cat(m.weights) / scale, cat(ctx.state_tensors("mom")) / scale] +
                   [cat(ctx.state_tensors("w_local", i)) / scale for i in range(K)])
        ctx.close()
    for a, b in zip(*res):
        assert np.array_equal(bits(a), bits(b))


def test_materialize_writes_out_recorded_state():
    """After a Pull iteration of ssd_step the w' arrays hold w_loc and w' is
    recorded as global; ssd_materialize must produce explicit arrays equal to
    the oracle's, and later fused steps must continue unchanged."""
    print("case: materialize", flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    numel, K, k, W = ODD, 3, 2, 1
    m = Model(numel, K, seed=21)
    ctx = B.Context(B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, chunk_elems=256,
                                  stream=torch.cuda.current_stream().cuda_stream), m.weights)
    o = Oracle(m.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    for it in range(W + 3 * k):
        ctx.ssd_step(m.g_dev[it % 3])
        o.step(m.g_host[it % 3])
        v = ctx.ssd_get_state()
        if it == W - 1:
            assert v.w_local_is_global == 1 and v.w_loc_where == B.SSD_W_LOC_IS_GLOBAL
        elif (it - W) % k == k - 1:
            assert v.w_local_is_global == 1 and v.w_loc_where == B.SSD_W_LOC_IN_W_LOCAL
        else:
            assert v.w_local_is_global == 0 and v.w_loc_where == B.SSD_W_LOC_IN_W_LOCAL
        if it in (W - 1, W + 1, W + 2):          # hand-over, a Pull iteration, a plain one
            ctx.ssd_materialize()
            v = ctx.ssd_get_state()
            assert v.w_local_is_global == 0
            torch.cuda.synchronize()
            for i in range(K):
                assert np.array_equal(bits(cat(ctx.state_tensors("w_local", i))), bits(o.wl[i])), it
                if v.w_loc_where == B.SSD_W_LOC_SEPARATE:
                    assert np.array_equal(bits(cat(ctx.state_tensors("w_loc", i))), bits(o.wloc[i])), it
        compare_state(ctx, m, o, exact=True, where="materialize it=%d" % it)
    ctx.close()


def test_mixed_fused_and_piecewise_iterations():
    """Alternate ssd_step with piecewise iterations inside one schedule; every
    hand-over between the two (recorded Pull -> explicit arrays) must keep the
    state equal to the oracle's."""
    print("case: mixed fused/piecewise", flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    numel, K, k, W = ODD, 3, 2, 2
    m = Model(numel, K, seed=31)
    ctx = B.Context(B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, chunk_elems=256,
                                  stream=torch.cuda.current_stream().cuda_stream), m.weights)
    o = Oracle(m.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    pattern = "FFFPFPPFFPFPFFPP"          # F: ssd_step, P: piecewise; first W are warm-up
    for it, how in enumerate(pattern):
        p = it % 3
        d = it - W
        if how == "F" or it < W:
            ctx.ssd_step(m.g_dev[p])
        else:
            ctx.ssd_server_aggregate_update(m.g_dev[p])
            for i in range(K):
                ctx.ssd_worker_glu_update(i, m.g_dev[p][i])
            if d % k == k - 1:
                for i in range(K):
                    ctx.ssd_worker_pull(i)
        o.step(m.g_host[p])
        if it >= W and how == "P":
            # piecewise iterations do not advance ssd_step's iteration counter;
            # the schedule is keyed on the local update count, which they do
            pass
        compare_state(ctx, m, o, exact=True, where="mixed it=%d %s" % (it, how))
    ctx.close()


@pytest.mark.parametrize("hp", [
    dict(lr=0.1, momentum=0.9, wd=1e-2, grad_sync_exact=1),                          # exact w_minus
    dict(lr=0.1, momentum=0.9, wd=1e-4, lr_loc=0.1, alpha=1.0, beta=0.0, wd_loc=0.0),  # plain local SGD
    dict(lr=0.1, momentum=0.9, wd=1e-4, alpha=0.0, beta=0.0),                        # pure decay
])
def test_local_updater_variants_bit_exact(hp):
    """Variants of the local updater the paper describes: grad_sync from the
    exact w_minus of Sec. 3.2.1; Eq. (worker) (alpha = 1, beta = 0, no decay);
    and the degenerate alpha = beta = 0."""
    print("case: local updater variant %r" % (hp,), flush=True)
    run_schedule(ODD, K=4, k=3, W=2, steps=2 + 8, hp=hp, seed=13,
                 lr_changes={6: (0.05, 0.2)} if hp.get("grad_sync_exact") else None)


def test_two_stream_schedule_of_fig_3b():
    """Server update on one stream, local updates (and Pulls) on another, with
    events only where Algorithm 1 has a data dependency: a Pull reads the
    global weight after this iteration's server update, and the next server
    update must not overwrite it before the Pulls have read it."""
    print("case: two streams", flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    numel, K, k, W = [70000, 513, 64, 1025], 4, 2, 1
    m = Model(numel, K, seed=41)
    main = torch.cuda.current_stream()
    s_srv, s_wrk = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = B.Context(B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, stream=main.cuda_stream), m.weights)
    o = Oracle(m.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    ctx.ssd_step(m.g_dev[0])                    # warm-up (also the last warm-up iteration)
    o.step(m.g_host[0])
    ctx.ssd_materialize()
    ready = torch.cuda.Event()
    ready.record(main)
    s_srv.wait_event(ready)
    s_wrk.wait_event(ready)
    pulls_done = None
    for d in range(3 * k + 1):
        p = (d + 1) % 3
        ctx.ssd_set_stream(s_srv)
        if pulls_done is not None:
            s_srv.wait_event(pulls_done)        # Pulls of the previous iteration read w
            pulls_done = None
        ctx.ssd_server_aggregate_update(m.g_dev[p])
        srv_done = torch.cuda.Event()
        srv_done.record(s_srv)
        ctx.ssd_set_stream(s_wrk)
        for i in range(K):
            ctx.ssd_worker_glu_update(i, m.g_dev[p][i])
        if d % k == k - 1:
            s_wrk.wait_event(srv_done)          # Pull w_t: after this iteration's server update
            for i in range(K):
                ctx.ssd_worker_pull(i)
            pulls_done = torch.cuda.Event()
            pulls_done.record(s_wrk)
        o.step(m.g_host[p])
        if d in (k, 3 * k):                     # elsewhere the two streams keep running freely
            torch.cuda.synchronize()
            compare_state(ctx, m, o, exact=True, where="two streams d=%d" % d)
    ctx.ssd_set_stream(main)
    ctx.close()


def test_multipliers_set_and_taken_back():
    """Without multipliers the kernels take the hyper-parameters from their
    arguments and ssd_set_lr uploads nothing; with multipliers they read the
    per-tensor table.  Going there and back (all multipliers 1 again, or NULL)
    with learning-rate changes on the way must leave the plain schedule's bits."""
    print("case: multipliers set and taken back", flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    numel, K, k, W = [3000, 257, 64], 3, 2, 1
    model = Model(numel, K, seed=77)
    ctx = B.Context(B.make_config(numel, K, k, W, 0.1, 0.9, 1e-3, stream=torch.cuda.current_stream().cuda_stream),
                    model.weights)
    o = Oracle(model.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-3, mode="f32")
    ones = [1.0] * len(numel)
    for it in range(W + 4 * k):
        if it == 2:
            ctx.ssd_set_tensor_multipliers(ones, ones)          # still uniform
        if it == 3:
            ctx.ssd_set_tensor_multipliers([1.0, 1.0, 1.0], [1.0, 1.0, 1.0 + 2.0 ** -23])
            ctx.ssd_set_tensor_multipliers(None, None)          # the table was uploaded, and is dropped again
        if it in (4, 6):
            lr, lr_loc = (0.05, 0.3) if it == 4 else (0.2, 0.6)
            ctx.ssd_set_lr(lr, lr_loc)
            o.set_lr(lr, lr_loc)
        ctx.ssd_step(model.g_dev[it % 3])
        o.step(model.g_host[it % 3])
        compare_state(ctx, model, o, exact=True, where="multipliers there and back it=%d" % it)
    ctx.close()


def test_per_tensor_multipliers_bit_exact():
    """lr / wd multipliers per tensor: every tensor must follow the oracle run
    with that tensor's own products (one binary32 multiplication each); a
    tensor with lr_mult = 0 stays frozen on the server and on the workers'
    side only decays by nothing (lr_loc = 0)."""
    print("case: per-tensor multipliers", flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    numel, K, k, W = ODD, 3, 2, 1
    lr, m_, wd = 0.1, 0.9, 1e-3
    lr_mult = [1.0, 0.5, 2.0, 0.0, 1.0, 0.25, 1.0, 3.0, 1.0, 0.0, 1.5, 1.0]
    wd_mult = [1.0, 0.0, 1.0, 1.0, 0.0, 2.0, 1.0, 1.0, 0.5, 0.0, 1.0, 0.0]
    model = Model(numel, K, seed=51)
    ctx = B.Context(B.make_config(numel, K, k, W, lr, m_, wd, grad_sync_exact=1,
                                  stream=torch.cuda.current_stream().cuda_stream), model.weights)
    ctx.ssd_set_tensor_multipliers(lr_mult, wd_mult)
    f = np.float32
    lr_loc = f(4.0) * f(lr)
    offs = np.concatenate([[0], np.cumsum(numel)])

    def oracle_for(t, lr_now, lr_loc_now):
        return dict(lr=float(f(lr_now) * f(lr_mult[t])), wd=float(f(wd) * f(wd_mult[t])),
                    lr_loc=float(f(lr_loc_now) * f(lr_mult[t])), wd_loc=float(f(wd) * f(wd_mult[t])))

    oracles = {}
    for t in range(len(numel)):
        if lr_mult[t] == 0.0:
            continue
        hp = oracle_for(t, lr, lr_loc)
        oracles[t] = Oracle(model.w0[offs[t]:offs[t + 1]], K=K, k=k, W=W, lr=hp["lr"], m=m_, wd=hp["wd"],
                            lr_loc=hp["lr_loc"], wd_loc=hp["wd_loc"], exact_w_minus=True, mode="f32")
    for it in range(W + 3 * k + 1):
        if it == W + 2:                    # a learning-rate change re-derives every tensor's values
            lr, lr_loc = 0.05, f(0.15)
            ctx.ssd_set_lr(lr, float(lr_loc))
            for t, o in oracles.items():
                hp = oracle_for(t, lr, lr_loc)
                o.set_lr(hp["lr"], hp["lr_loc"])
        p = it % 3
        ctx.ssd_step(model.g_dev[p])
        for t, o in oracles.items():
            o.step([g[offs[t]:offs[t + 1]] for g in model.g_host[p]])
        torch.cuda.synchronize()
        v = ctx.ssd_get_state()
        mom = ctx.state_tensors("mom")
        for t in range(len(numel)):
            w_t = model.weights[t].cpu().numpy()
            if t not in oracles:           # frozen
                assert np.array_equal(w_t, model.w0[offs[t]:offs[t + 1]]), (it, t)
                assert not np.any(mom[t].cpu().numpy()), (it, t)
                if v.has_local and not v.w_local_is_global:
                    for i in range(K):
                        wl = ctx.state_tensors("w_local", i)[t].cpu().numpy()
                        assert np.array_equal(wl, w_t), (it, t, i)
                continue
            o = oracles[t]
            assert np.array_equal(bits(w_t), bits(o.w)), (it, t, "w")
            assert np.array_equal(bits(mom[t]), bits(o.mom)), (it, t, "mom")
            if v.has_local and not v.w_local_is_global:
                for i in range(K):
                    wl = ctx.state_tensors("w_local", i)[t]
                    assert np.array_equal(bits(wl), bits(o.wloc[i] if v.w_local_is_global else o.wl[i])), (it, t, i)
            elif v.has_local and v.w_loc_where == B.SSD_W_LOC_IN_W_LOCAL:
                for i in range(K):
                    assert np.array_equal(bits(ctx.state_tensors("w_local", i)[t]), bits(o.wloc[i])), (it, t, i)
            if o.d > 0:
                assert np.array_equal(bits(ctx.state_tensors("pre")[t]), bits(o.pre[0])), (it, t, "pre")
    ctx.close()


@pytest.mark.parametrize("seed", range(24))
def test_randomized_configurations(seed):
    """Seeded random draws over the whole configuration space: worker count,
    delay, warm-up length, tensor sizes (tiny, ragged, multi-block), pointer
    misalignment, hyper-parameters, the exact-w_minus variant, chunk size."""
    rng = np.random.default_rng(1000 + seed)
    K = int(rng.integers(1, 17))
    k = int(rng.integers(0, 7))
    W = int(rng.integers(0, 4))
    T = int(rng.integers(1, 9))
    numel = [int(x) for x in rng.choice([1, 2, 3, 4, 5, 7, 64, 255, 256, 257, 511, 513, 1000, 1024, 1025, 3000, 5001],
                                        size=T)]
    hp = dict(lr=float(rng.choice([0.01, 0.1, 0.5])), momentum=float(rng.choice([0.0, 0.5, 0.9])),
              wd=float(rng.choice([0.0, 1e-4, 1e-2])), alpha=float(rng.choice([0.0, 1.0, 2.0])),
              beta=float(rng.choice([0.0, 0.5, 1.0])), grad_sync_exact=int(rng.integers(0, 2)))
    if rng.random() < 0.5:
        hp["lr_loc"] = float(rng.choice([0.05, 0.4, 1.6]))
    if rng.random() < 0.5:
        hp["wd_loc"] = float(rng.choice([0.0, 1e-3]))
    if rng.random() < 0.3:
        hp["rescale_grad"] = float(rng.choice([1.0, 0.25]))
    w_shift = int(rng.choice([0, 0, 1, 2]))
    g_shift = int(rng.choice([0, 0, 1, 3]))
    chunk = int(rng.choice([0, 256, 512, 1024]))
    steps = W + (2 * k + 2 if k else 4)
    print("case: random seed=%d K=%d k=%d W=%d numel=%r hp=%r shifts=%d/%d chunk=%d" % (
        seed, K, k, W, numel, hp, w_shift, g_shift, chunk), flush=True)
    run_schedule(numel, K=K, k=k, W=W, steps=steps, hp=hp, seed=seed, w_shift=w_shift, g_shift=g_shift,
                 chunk_elems=chunk)


@pytest.mark.parametrize("seed", range(24))
def test_randomized_configurations_with_lead_ins_and_gradient_types(seed):
    """Seeded random draws over everything a configuration can combine: worker
    count (planar and interleaved local weights), delay, warm-up length, tensor
    sizes around the tile, lead-in and block boundaries, pointer misalignment,
    block size, gradient element type, exact w_minus, hyper-parameters and a
    learning-rate change -- each against the oracle, bit for bit, with both
    cache policies side by side."""
    rng = np.random.default_rng(2000 + seed)
    K = int(rng.choice([1, 2, 3, 5, 7, 8, 9, 10, 13, 16]))
    k = int(rng.choice([1, 2, 3, 5]))
    W = int(rng.choice([0, 1, 2]))
    sizes = [int(rng.choice([1, 3, 4, 63, 255, 256, 257, 1000, 4099, 8191, 8192, 8193, 9000, 20001]))
             for _ in range(int(rng.integers(1, 7)))]
    w_shift = int(rng.choice([0, 0, 0, 1, 4, 8]))
    g_shift = int(rng.choice([0, 0, 0, 2, 4, 12]))
    chunk = int(rng.choice([0, 256, 512, 1024]))
    gd = int(rng.choice([0, 0, 1, 2]))
    if gd:                       # 16-bit buffers: shifts in elements of 2 bytes, keep them even for 4-byte alignment
        g_shift -= g_shift % 2
    hp = dict(lr=float(rng.choice([0.1, 0.05])), momentum=float(rng.choice([0.9, 0.5])), wd=float(rng.choice([1e-4, 0.0])),
              alpha=float(rng.choice([2.0, 1.0])), beta=float(rng.choice([0.5, 0.25])),
              grad_sync_exact=int(rng.integers(0, 2)))
    steps = W + 2 * k + int(rng.integers(1, 4))
    lr_changes = {int(rng.integers(1, steps)): (0.03, 0.2)} if rng.integers(0, 2) else None
    print("case: random (lead-ins, types) seed=%d K=%d k=%d W=%d sizes=%s w_shift=%d g_shift=%d chunk=%d gd=%d hp=%s lr_changes=%s"
          % (seed, K, k, W, sizes, w_shift, g_shift, chunk, gd, hp, lr_changes), flush=True)
    run_schedule(sizes, K=K, k=k, W=W, steps=steps, hp=hp, chunk_elems=chunk, seed=seed, w_shift=w_shift,
                 g_shift=g_shift, grad_dtype=gd, lr_changes=lr_changes, P=2)
