"""GPU parity: the HIP library against the CPU oracle, through the C ABI.

Bit-exact against the binary32 oracle (same rounding sequence), and within
1e-5 (per tensor, max |a-b| / max |b|) against the binary64 oracle."""
import numpy as np
import pytest
import torch

from ssd_harness import Model, bits, cat, compare_state, effective_w_loc, run_schedule

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
    for ce in (1024, 2048, 8192, 0):
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
    ca = B.Context(B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, stream=s, chunk_elems=1024), ma.weights)
    cb = B.Context(B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, stream=s, chunk_elems=1024), mb.weights)
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
                assert np.array_equal(bits(cat(ca.state_tensors("w_local", i))),
                                      bits(cat(cb.state_tensors("w_local", i)))), (it, i)
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
        torch.cuda.synchronize()
        res.append([cat(m.weights) / scale, cat(ctx.state_tensors("mom")) / scale] +
                   [cat(ctx.state_tensors("w_local", i)) / scale for i in range(K)])
        ctx.close()
    for a, b in zip(*res):
        assert np.array_equal(bits(a), bits(b))
