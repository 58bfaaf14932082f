"""GPU parity with 16-bit gradient buffers (bfloat16, binary16): an extension
beyond the paper, whose gradients are binary32.

A 16-bit gradient is a binary32 value; the library widens it exactly while
loading and then runs the same binary32 sequence.  The oracle is therefore
unchanged: it is fed the same gradient values as float32 arrays, and the
results must agree bit for bit.  The widening itself is checked on every one
of the 65 536 bit patterns of each type against numpy's conversions."""
import numpy as np
import pytest
import torch

from ssd_harness import Model, bits, cat, compare_state, effective_w_loc, effective_w_local, run_schedule

pytestmark = pytest.mark.gpu

ODD = [1, 3, 4, 5, 63, 64, 65, 1023, 1024, 1025, 4097, 2051]
BF16, F16 = 1, 2
NAMES = {BF16: "bf16", F16: "f16"}


def widen_all_patterns(gd):
    """float32 values of the 16-bit patterns 0 .. 65535, by numpy alone."""
    u = np.arange(65536, dtype=np.uint32)
    if gd == BF16:
        return (u << 16).astype(np.uint32).view(np.float32)
    return u.astype(np.uint16).view(np.float16).astype(np.float32)


@pytest.mark.parametrize("gd", [BF16, F16])
@pytest.mark.parametrize("shift", [0, 1, 4])
def test_every_16bit_pattern_is_widened_exactly(gd, shift):
    """K = 1, rescale = 1, lr = 1, m = 0, wd = 0, w = 0: the server update
    gives mom' = -g, w' = -g, so each state array shows the widened gradient.
    shift: elements by which the gradient buffer is displaced (1: two-byte
    alignment, element-wise path; 4: eight-byte alignment, 64-bit loads)."""
    print("case: all patterns %s shift=%d" % (NAMES[gd], shift), flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    n = 65536
    tdt = B.GRAD_TORCH_DTYPE[gd]
    patterns = torch.from_numpy(np.arange(n, dtype=np.uint16).view(np.int16))
    buf = torch.zeros(n + 8, dtype=torch.int16, device="cuda")
    buf[shift:shift + n] = patterns.cuda()
    g = buf.view(tdt)[shift:shift + n]
    w = torch.zeros(n, dtype=torch.float32, device="cuda")
    cfg = B.make_config([n], 1, 0, 0, lr=1.0, momentum=0.0, wd=0.0, rescale_grad=1.0,
                        stream=torch.cuda.current_stream().cuda_stream, grad_dtype=gd)
    ctx = B.Context(cfg, [w])
    ctx.ssd_step([[g]])
    torch.cuda.synchronize()
    wide = widen_all_patterns(gd)
    got_w = w.cpu().numpy()
    got_m = ctx.state_tensors("mom")[0].cpu().numpy()
    fin = np.isfinite(wide) & (wide != 0)
    assert np.array_equal(bits(got_w[fin]), bits(-wide[fin]))
    assert np.array_equal(bits(got_m[fin]), bits(-wide[fin]))
    assert np.array_equal(np.isnan(got_w), np.isnan(wide))
    assert np.array_equal(np.isinf(got_w), np.isinf(wide))
    # and the whole array, zeros and infinities included, against the oracle
    o = Oracle(np.zeros(n, np.float32), K=1, k=0, W=0, lr=1.0, m=0.0, wd=0.0, rescale=1.0, mode="f32")
    with np.errstate(all="ignore"):
        o.step([wide])
    both_nan = np.isnan(got_w) & np.isnan(o.w)
    assert np.all((bits(got_w) == bits(o.w)) | both_nan)
    ctx.close()


@pytest.mark.parametrize("gd", [BF16, F16])
@pytest.mark.parametrize("K", [1, 2, 3, 5, 8, 16])
def test_odd_tensors_bit_exact(gd, K):
    print("case: %s odd tensors K=%d" % (NAMES[gd], K), flush=True)
    run_schedule(ODD, K=K, k=3, W=2, steps=2 + 7, seed=K, grad_dtype=gd)


@pytest.mark.parametrize("gd", [BF16, F16])
@pytest.mark.parametrize("k,W", [(0, 2), (1, 0), (2, 1), (4, 2)])
def test_schedules_bit_exact(gd, k, W):
    print("case: %s schedule k=%d W=%d" % (NAMES[gd], k, W), flush=True)
    run_schedule(ODD, K=4, k=k, W=W, steps=W + 3 * max(k, 1) + 1, seed=10 * k + W, grad_dtype=gd)


@pytest.mark.parametrize("gd", [BF16, F16])
@pytest.mark.parametrize("w_shift,g_shift", [(0, 1), (0, 2), (0, 4), (1, 4), (3, 3)])
def test_alignments(gd, w_shift, g_shift):
    """g_shift 1, 2, 3: below the 8 bytes one 64-bit load needs; 4: exactly 8."""
    print("case: %s w_shift=%d g_shift=%d" % (NAMES[gd], w_shift, g_shift), flush=True)
    run_schedule(ODD, K=3, k=2, W=1, steps=6, w_shift=w_shift, g_shift=g_shift, seed=5, grad_dtype=gd)


@pytest.mark.parametrize("gd", [BF16, F16])
def test_remaining_worker_counts_and_chunks(gd):
    for K in (4, 6, 7, 9, 10, 11, 12, 13, 14, 15):
        print("case: %s K=%d" % (NAMES[gd], K), flush=True)
        run_schedule([5000, 17], K=K, k=2, W=1, steps=5, seed=K, grad_dtype=gd,
                     chunk_elems=(0, 512, 1024)[K % 3])


@pytest.mark.parametrize("gd", [BF16, F16])
@pytest.mark.parametrize("K,w_shift,g_shift", [(3, 0, 0), (12, 0, 4), (2, 4, 2)])
def test_lead_in_of_large_tensors(gd, K, w_shift, g_shift):
    """Tensors of 32 tiles and more start inside their first arena block (the
    tiles follow the weight pointer's 1 KiB grid); 16-bit gradients at the
    same element offsets, at 8-byte and at 4-byte alignment."""
    print("case: %s lead-in K=%d w_shift=%d g_shift=%d" % (NAMES[gd], K, w_shift, g_shift), flush=True)
    run_schedule([9000, 8192 + 3, 64, 10001, 20000, 5], K=K, k=2, W=1, steps=6, w_shift=w_shift, g_shift=g_shift,
                 seed=40 + K, grad_dtype=gd)


@pytest.mark.parametrize("gd", [BF16, F16])
def test_variants_and_plain_oracle(gd):
    print("case: %s variants" % NAMES[gd], flush=True)
    hp = dict(lr=0.05, momentum=0.8, wd=1e-3, lr_loc=0.3, alpha=1.5, beta=0.25, wd_loc=2e-3,
              rescale_grad=0.125, grad_sync_exact=1)
    run_schedule(ODD, K=4, k=2, W=2, steps=9, hp=hp, seed=3, grad_dtype=gd,
                 lr_changes={4: (0.02, 0.1), 7: (0.2, 0.8)})
    run_schedule([30000, 513, 64], K=8, k=4, W=2, steps=2 + 20, mode="f64", check_every=22, seed=9,
                 grad_dtype=gd)


def test_loss_scaled_f16_gradients_overflow_like_ieee():
    """binary16 gradients near and beyond the type's range (a loss scale that
    is too large): +-inf and NaN must come through as they do in the oracle."""
    print("case: f16 overflow", flush=True)
    with np.errstate(all="ignore"):
        run_schedule([3000, 7], K=2, k=2, W=1, steps=5, g_scale=3e4, seed=11, grad_dtype=F16,
                     hp=dict(lr=0.1, momentum=0.9, wd=1e-4, rescale_grad=1.0 / 1024))


@pytest.mark.parametrize("gd", [BF16, F16])
def test_piecewise_calls_equal_fused_step(gd):
    """server + K x glu (+ K x pull) == ssd_step with 16-bit gradients too."""
    print("case: %s piecewise" % NAMES[gd], flush=True)
    from oracle.ssd_oracle import Oracle
    from paper_2012_05396_amd import binding as B
    numel, K, k, W = ODD, 3, 2, 1
    tdt = B.GRAD_TORCH_DTYPE[gd]
    ma = Model(numel, K, seed=78, grad_dtype=tdt, g_shift=4)
    mb = Model(numel, K, seed=78, grad_dtype=tdt, g_shift=1)
    s = torch.cuda.current_stream().cuda_stream
    mk = lambda: B.make_config(numel, K, k, W, 0.1, 0.9, 1e-4, stream=s, grad_dtype=gd)
    ca, cb = B.Context(mk(), ma.weights), B.Context(mk(), mb.weights)
    o = Oracle(ma.w0, K=K, k=k, W=W, lr=0.1, m=0.9, wd=1e-4, mode="f32")
    for it in range(W + 3 * k + 1):
        p = it % 3
        ca.ssd_step(ma.g_dev[p])
        o.step(ma.g_host[p])
        cb.ssd_server_aggregate_update(mb.g_dev[p])
        if it == W - 1:
            for i in range(K):
                cb.ssd_worker_pull(i)
        elif it >= W:
            for i in range(K):
                cb.ssd_worker_glu_update(i, mb.g_dev[p][i])
            if (it - W) % k == k - 1:
                for i in range(K):
                    cb.ssd_worker_pull(i)
        compare_state(ca, ma, o, exact=True, where="%s fused it=%d" % (NAMES[gd], it))
        compare_state(cb, mb, o, exact=True, where="%s piecewise it=%d" % (NAMES[gd], it))
        for i in range(K):
            assert np.array_equal(bits(effective_w_local(ca, ma, i)), bits(effective_w_local(cb, mb, i)))
            assert np.array_equal(bits(effective_w_loc(ca, ma, i)), bits(effective_w_loc(cb, mb, i)))
    ca.close(); cb.close()


def test_binding_refuses_buffers_of_another_type():
    """The C ABI sees raw pointers; the binding knows the tensors and must not
    let a float32 buffer through to a 16-bit context or the reverse."""
    from paper_2012_05396_amd import binding as B
    n = 1000
    s = torch.cuda.current_stream().cuda_stream
    w = torch.zeros(n, device="cuda")
    g32 = torch.zeros(n, device="cuda")
    g16 = torch.zeros(n, device="cuda", dtype=torch.bfloat16)
    c16 = B.Context(B.make_config([n], 1, 0, 0, 0.1, 0.9, 0.0, stream=s, grad_dtype=BF16), [w])
    c32 = B.Context(B.make_config([n], 1, 0, 0, 0.1, 0.9, 0.0, stream=s), [w])
    with pytest.raises(B.SsdError):
        c16.ssd_step([[g32]])
    with pytest.raises(B.SsdError):
        c32.ssd_step([[g16]])
    with pytest.raises(B.SsdError):
        c16.ssd_step([[g16[:n - 1]]])
    with pytest.raises(B.SsdError):
        B.Context(B.make_config([n], 1, 0, 0, 0.1, 0.9, 0.0, stream=s, grad_dtype=3), [w])
    c16.close(); c32.close()
