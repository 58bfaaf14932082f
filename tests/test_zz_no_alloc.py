"""The allocation-free entry point, ssd_server_aggregate_update_noalloc,
against the context-based ssd_server_aggregate_update (and the oracle) through
the C ABI: bit-identical weights and momentum on calls that follow each other
on one GPU, the later ones with smaller inputs, so that whatever an earlier
call left in the library's static device array must not leak into a later
result.  Named so that pytest collects it last."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2012_05396_amd import binding as B


def _clone_views(model):
    """A second copy of the model's weight buffer with the same layout."""
    flat = model.wflat.clone()
    base = model.wflat.data_ptr()
    views = []
    for w in model.weights:
        o = (w.data_ptr() - base) // 4
        views.append(flat[o:o + w.numel()])
    return flat, views


def _run_case(sizes, K, iters, seed, w_shift=0, g_shift=0, hp=(0.1, 0.9, 1e-4)):
    from oracle.ssd_oracle import Oracle
    from ssd_harness import Model, bits, cat
    lr, m, wd = hp
    model = Model(sizes, K, P=iters, seed=seed, w_shift=w_shift, g_shift=g_shift)
    w2flat, w2 = _clone_views(model)
    mom2flat = torch.zeros_like(w2flat)
    base = w2flat.data_ptr()
    mom2 = [mom2flat[(w.data_ptr() - base) // 4:(w.data_ptr() - base) // 4 + w.numel()] for w in w2]
    stream = torch.cuda.current_stream().cuda_stream
    ctx = B.Context(B.make_config(sizes, K, 0, 0, lr, m, wd, stream=stream), model.weights)
    o = Oracle(model.w0, K=K, k=0, W=0, lr=lr, m=m, wd=wd, mode="f32")
    rescale = ctx.cfg.rescale_grad
    for it in range(iters):
        ctx.ssd_server_aggregate_update(model.g_dev[it])
        B.ssd_server_aggregate_update_noalloc(w2, mom2, model.g_dev[it], lr, m, wd, rescale, stream=stream)
        o.server(model.g_host[it])
        torch.cuda.synchronize()
        tag = "sizes=%s K=%d it=%d" % (sizes[:3], K, it)
        assert np.array_equal(bits(cat(w2)), bits(cat(model.weights))), "weights differ: " + tag
        assert np.array_equal(bits(cat(mom2)), bits(cat(ctx.state_tensors("mom")))), "momentum differs: " + tag
        assert np.array_equal(bits(cat(w2)), bits(o.w)) and np.array_equal(bits(cat(mom2)), bits(o.mom)), tag
    # nothing outside the tensors was written
    inside = torch.zeros_like(w2flat, dtype=torch.bool)
    for v in w2:
        o0 = (v.data_ptr() - base) // 4
        inside[o0:o0 + v.numel()] = True
    assert torch.equal(w2flat[~inside], model.wflat[~inside]) and not mom2flat[~inside].any()
    ctx.close()


@pytest.mark.gpu
def test_noalloc_server_update_equals_the_context_entry_point():
    print("case: no-alloc entry point, calls in a row with shrinking inputs", flush=True)
    # several tiles, ragged tails, a tensor of one element; then smaller models
    _run_case([70000, 4097, 1025, 1024, 64, 5, 1], K=5, iters=2, seed=1)
    _run_case([3000, 63], K=3, iters=2, seed=2)
    _run_case([257], K=1, iters=1, seed=3)
    # tensors whose pointers are not 16-byte aligned take the scalar path
    _run_case([2051, 1023, 4], K=2, iters=1, seed=4, w_shift=1, g_shift=3)
    # many tensors: the records travel in several launches (22 per launch at K = 16)
    _run_case([300 + 7 * t for t in range(60)], K=16, iters=1, seed=5)


@pytest.mark.gpu
def test_noalloc_randomized_cases():
    """Seeded random shapes, worker counts, alignments and hyper-parameters,
    one after the other on the same static array."""
    print("case: no-alloc entry point, randomized", flush=True)
    rng = np.random.default_rng(2024)
    for case in range(8):
        T = int(rng.integers(1, 40))
        sizes = [int(x) for x in rng.integers(1, 6000, size=T)]
        K = int(rng.integers(1, 17))
        hp = (float(rng.choice([0.05, 0.1, 1.0])), float(rng.choice([0.0, 0.5, 0.9])), float(rng.choice([0.0, 1e-4, 1e-2])))
        _run_case(sizes, K=K, iters=2, seed=50 + case, w_shift=int(rng.integers(0, 4)),
                  g_shift=int(rng.integers(0, 4)), hp=hp)


def _args(K=2, T=2, numel=(10, 20)):
    n = (C.c_int64 * T)(*numel)
    w = (C.c_void_p * T)(*[0x10000 * (t + 1) for t in range(T)])
    mo = (C.c_void_p * T)(*[0x900000 + 0x10000 * t for t in range(T)])
    rows = [(C.c_void_p * T)(*[0x2000000 + 0x100000 * i + 0x1000 * t for t in range(T)]) for i in range(K)]
    g = (C.c_void_p * K)(*[C.cast(r, C.c_void_p).value for r in rows])
    return n, w, mo, g, rows


def test_noalloc_rejects_bad_arguments_before_touching_a_device():
    f = B.lib.ssd_server_aggregate_update_noalloc
    hp = (0.1, 0.9, 1e-4, 0.5, 0, None)
    n, w, mo, g, rows = _args()
    assert f(0, 2, n, w, mo, g, *hp) == B.SSD_EINVAL
    assert f(17, 2, n, w, mo, g, *hp) == B.SSD_EINVAL
    assert f(2, 0, n, w, mo, g, *hp) == B.SSD_EINVAL
    assert f(2, 2, None, w, mo, g, *hp) == B.SSD_EINVAL
    assert f(2, 2, n, None, mo, g, *hp) == B.SSD_EINVAL
    assert f(2, 2, n, w, None, g, *hp) == B.SSD_EINVAL
    assert f(2, 2, n, w, mo, None, *hp) == B.SSD_EINVAL
    assert f(2, 2, n, w, mo, g, 0.1, 0.9, 1e-4, 0.5, -1, None) == B.SSD_EINVAL
    # sizes beyond what the static scratch holds
    assert f(2, B.SSD_NOALLOC_MAX_TENSORS + 1, n, w, mo, g, *hp) == B.SSD_EINVAL
    assert b"static scratch" in B.lib.ssd_last_error(None)
    big = (C.c_int64 * 2)(256 * B.SSD_NOALLOC_MAX_BLOCKS, 1)
    assert f(2, 2, big, w, mo, g, *hp) == B.SSD_EINVAL
    assert b"static scratch" in B.lib.ssd_last_error(None)
    huge = (C.c_int64 * 2)(2 ** 62, 2 ** 62)
    assert f(2, 2, huge, w, mo, g, *hp) == B.SSD_EINVAL
    zero = (C.c_int64 * 2)(10, 0)
    assert f(2, 2, zero, w, mo, g, *hp) == B.SSD_EINVAL
    # NULL and misaligned pointers
    n, w, mo, g, rows = _args()
    w[1] = None
    assert f(2, 2, n, w, mo, g, *hp) == B.SSD_EINVAL
    n, w, mo, g, rows = _args()
    mo[0] = mo[0] + 2
    assert f(2, 2, n, w, mo, g, *hp) == B.SSD_EALIGN
    n, w, mo, g, rows = _args()
    rows[1][1] = rows[1][1] + 1
    assert f(2, 2, n, w, mo, g, *hp) == B.SSD_EALIGN
    n, w, mo, g, rows = _args()
    rows[0][0] = None
    assert f(2, 2, n, w, mo, g, *hp) == B.SSD_EINVAL
