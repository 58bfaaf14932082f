"""Full-size GPU parity on the five benchmark configurations, in the launch
configuration bench.py times (library defaults: 256-element chunks, measured
waves-per-CU caps).

The path is element-wise, so the oracle can compute any element on its own:
a seeded sample of elements of every tensor (first and last elements, both
sides of chunk boundaries, random positions) is gathered from the inputs, run
through the CPU oracle for the whole schedule, and compared bit for bit
(binary32 oracle) and within 1e-5 per element (binary64 oracle; relative to
the element, with a floor of a tenth of its tensor's largest value) with the same elements of
the GPU state, after each of the last iterations so that every kernel variant
is covered.  Properties that hold at any size are checked on whole arrays on
the device: pre_weight equals the global weight as of the last Pull, and the
fused step equals the piecewise calls on every element.
"""
import numpy as np
import pytest
import torch

from oracle.ssd_oracle import Oracle
from paper_2012_05396_amd import workloads

pytestmark = pytest.mark.gpu

SAMPLES_PER_TENSOR = 2048
EXTRA_INDICES = {}   # tensor index -> more element indices to check


def sample_indices(numel, chunk, rng):
    """Element indices inside one tensor worth checking."""
    idx = set(range(min(numel, 8))) | set(range(max(0, numel - 8), numel))
    nchunks = -(-numel // chunk)
    for c in rng.choice(nchunks, size=min(nchunks, 6), replace=False):
        for e in (c * chunk - 1, c * chunk, c * chunk + 1, c * chunk + 3, c * chunk + 4,
                  c * chunk + chunk - 1):
            if 0 <= e < numel:
                idx.add(int(e))
    if numel > len(idx):
        idx |= set(int(x) for x in rng.integers(0, numel, size=min(SAMPLES_PER_TENSOR, numel)))
    return np.array(sorted(idx), np.int64)


def bit_equal(a, b):
    a, b = np.asarray(a, np.float32), np.asarray(b, np.float32)
    return np.array_equal(a.view(np.int32), b.view(np.int32))


def run_full(name, piecewise_check=False, wl=None, grad_dtype=0, tol_elem=1e-5):
    """grad_dtype: an ssd_grad_dtype; with a 16-bit type the generator rounds
    the drawn gradients to it and the oracle gets those values as float32."""
    from paper_2012_05396_amd import binding as B
    wl = wl or workloads.workload(name)
    dev = torch.device("cuda", 0)
    numel = workloads.numels(wl.tensors)
    T, K, k, W = len(numel), wl.K, wl.k, wl.W
    steps = W + wl.steps
    print("case: %s N=%d T=%d K=%d k=%d steps=%d grad_dtype=%d" % (name, sum(numel), T, K, k, steps, grad_dtype),
          flush=True)
    rng = np.random.default_rng(wl.seed)

    wflat, offs = workloads.initial_weights(wl, device=dev)
    weights = workloads.views(wflat, wl.tensors, offs)
    P = 2
    gsets = [workloads.gradient_set(wl, p, device=dev, dtype=B.GRAD_TORCH_DTYPE[grad_dtype]) for p in range(P)]
    gviews = [[workloads.views(g, wl.tensors, offs) for g in gs] for gs in gsets]
    tables = [B.GradTable(g) for g in gviews]
    stream = torch.cuda.current_stream().cuda_stream
    mk = lambda: B.make_config(numel, K, k, W, wl.lr, wl.momentum, wl.wd, stream=stream, grad_dtype=grad_dtype)
    ctx = B.Context(mk(), weights)
    v = ctx.ssd_get_state()
    assert v.chunk_elems == 256
    # the library's own choice of cache policy: ordinary accesses while one iteration's arrays fit 256 MiB
    touched = v.num_chunks * v.chunk_elems * (K * (4 if grad_dtype == 0 else 2) + 4 * (K + 3))
    assert v.streaming == (1 if touched > 256 << 20 else 0) and (v.streaming == 1 or sum(numel) < 2_000_000)

    # sample: indices into the caller's flat buffers and into the arena
    flat_idx, arena_idx, seg_start, seg_len = [], [], [], []
    for t in range(T):
        idx = sample_indices(numel[t], v.chunk_elems, rng)
        if t in EXTRA_INDICES:
            idx = np.unique(np.concatenate([idx, EXTRA_INDICES[t].astype(np.int64)]))
        seg_start.append(sum(seg_len))
        seg_len.append(idx.size)
        flat_idx.append(idx + offs[t])
        arena_idx.append(idx + v.tensor_offset[t])
    flat_idx = torch.from_numpy(np.concatenate(flat_idx)).to(dev)
    arena_idx = torch.from_numpy(np.concatenate(arena_idx)).to(dev)
    S = flat_idx.numel()
    take = lambda flat, idx: flat.index_select(0, idx).to(torch.float32).cpu().numpy()
    w0 = take(wflat, flat_idx)
    gh = [[take(g, flat_idx) for g in gs] for gs in gsets]
    oracles = [Oracle(w0, K=K, k=k, W=W, lr=wl.lr, m=wl.momentum, wd=wl.wd, mode=m)
               for m in ("f32", "f64")]

    ctx2 = None
    if piecewise_check:
        w2 = wflat.clone()
        ctx2 = B.Context(mk(), workloads.views(w2, wl.tensors, offs))

    def arena(which, worker=0):
        return ctx.state_array(which, worker)

    def check(it):
        """Compare the sample with both oracles, and whole-array properties."""
        # ---- compare the sample with both oracles ----
        torch.cuda.synchronize()
        vv = ctx.ssd_get_state()
        o32, o64 = oracles
        got = {"w": take(wflat, flat_idx), "mom": take(arena("mom"), arena_idx)}
        exp32 = {"w": o32.w, "mom": o32.mom}
        exp64 = {"w": o64.w, "mom": o64.mom}
        if k > 0 and vv.has_local:
            for i in range(K):
                wl_i = got["w"] if vv.w_local_is_global else take(arena("w_local", i), arena_idx)
                got["w_local%d" % i] = wl_i
                exp32["w_local%d" % i], exp64["w_local%d" % i] = o32.wl[i], o64.wl[i]
                if vv.w_loc_where == B.SSD_W_LOC_IS_GLOBAL:
                    wloc_i = got["w"]
                elif vv.w_loc_where == B.SSD_W_LOC_IN_W_LOCAL:
                    wloc_i = take(arena("w_local", i), arena_idx)
                else:
                    wloc_i = take(arena("w_loc", i), arena_idx)
                got["w_loc%d" % i] = wloc_i
                exp32["w_loc%d" % i], exp64["w_loc%d" % i] = o32.wloc[i], o64.wloc[i]
            if o32.d > 0:
                got["pre"] = take(arena("pre"), arena_idx)
                exp32["pre"], exp64["pre"] = o32.pre[0], o64.pre[0]
        for name_, g in got.items():
            assert bit_equal(g, exp32[name_]), "%s it=%d %s: sampled elements differ from the binary32 oracle" % (
                name, it, name_)
            # per element: |a-b| / max(|b|, 0.1 * max|b| over the element's tensor)
            e = np.asarray(exp64[name_], np.float64)
            tmax = np.maximum.reduceat(np.abs(e), seg_start)
            floor = np.maximum(np.repeat(0.1 * tmax, seg_len), 1e-30)
            diff = np.abs(g.astype(np.float64) - e)
            err = np.max(diff / np.maximum(np.abs(e), floor))
            assert err <= tol_elem, "%s it=%d %s: per-element rel err %.3e vs binary64 oracle" % (name, it, name_, err)
            # per tensor: max|a-b| / max|b|
            err_t = np.max(np.maximum.reduceat(diff, seg_start) / np.maximum(tmax, 1e-30))
            assert err_t <= 1e-5, "%s it=%d %s: per-tensor rel err %.3e vs binary64 oracle" % (name, it, name_, err_t)
        # ---- whole-array properties, on the device ----
        if k > 0 and o32.d > 0 and (o32.d - 1) % k == 0 and o32.d > 1 and last_pull_w is not None:
            # pre_weight was just refreshed: it is the global weight of the previous Pull
            pre = arena("pre")
            for t in range(T):
                a = pre[vv.tensor_offset[t]:vv.tensor_offset[t] + numel[t]]
                b = last_pull_w[offs[t]:offs[t] + numel[t]]
                assert torch.equal(a.view(torch.int32), b.view(torch.int32)), (name, it, t)

    last_pull_w = None      # global weight as of the last Pull / hand-over
    for it in range(steps):
        p = it % P
        ctx.ssd_step(tables[p])
        kinds = [o.step(gh[p]) for o in oracles]
        if ctx2 is not None:
            ctx2.ssd_server_aggregate_update(tables[p])
            if kinds[0] == 1:
                for i in range(K):
                    ctx2.ssd_worker_pull(i)
            elif kinds[0] >= 2:
                for i in range(K):
                    ctx2.ssd_worker_glu_update(i, gviews[p][i])
                if kinds[0] == 3:
                    for i in range(K):
                        ctx2.ssd_worker_pull(i)
        if it >= steps - (k + 2) or it == W:
            check(it)
        if kinds[0] in (1, 3):
            last_pull_w = wflat.clone()
    if ctx2 is not None:
        # the fused step equals the piecewise calls on every element
        ctx.ssd_materialize()
        torch.cuda.synchronize()
        assert torch.equal(wflat.view(torch.int32), w2.view(torch.int32))
        va, vb = ctx.ssd_get_state(), ctx2.ssd_get_state()
        for which, cnt in (("mom", 1), ("pre", 1), ("w_local", K)):
            if k == 0 and which != "mom":
                continue
            for i in range(cnt):
                a, b = ctx.state_array(which, i), ctx2.state_array(which, i)
                for t in range(T):
                    # each context has its own arena offsets (they follow its weight pointers)
                    sa = slice(va.tensor_offset[t], va.tensor_offset[t] + numel[t])
                    sb = slice(vb.tensor_offset[t], vb.tensor_offset[t] + numel[t])
                    assert torch.equal(a[sa].view(torch.int32), b[sb].view(torch.int32)), (name, which, i, t)
    ctx.close()
    if ctx2 is not None:
        ctx2.close()
    del gsets, gviews, tables, wflat
    torch.cuda.empty_cache()
    return S



@pytest.mark.parametrize("name", ["resnet20", "resnet56", "resnet50", "vgg16", "resnet152_k2",
                                  "resnet152_k4", "resnet152_k8", "alexnet", "vgg11"])
def test_full_size_sampled_parity(name):
    run_full(name)


@pytest.mark.parametrize("name", ["resnet56", "resnet50"])
def test_full_size_fused_equals_piecewise_everywhere(name):
    run_full(name, piecewise_check=True)


@pytest.mark.parametrize("name,gd", [("resnet56", 1), ("vgg16", 1), ("resnet152_k4", 1), ("vgg16", 2),
                                     ("resnet50", 2)])
def test_full_size_sampled_parity_16bit_gradients(name, gd):
    """Extension beyond the paper: bfloat16 (1) / binary16 (2) gradient buffers."""
    run_full(name, grad_dtype=gd, piecewise_check=(name == "resnet50"))


@pytest.mark.parametrize("name,gd", [("vgg16", 0), ("resnet152_k4", 0), ("vgg16", 1), ("resnet50", 0),
                                     ("resnet152_k8", 0), ("resnet152_k2", 1)])
def test_every_element_bit_exact_at_full_size(name, gd):
    """The 138 M-element benchmark configuration (also with bfloat16 gradient
    buffers), the 25.6 M-element one and the K = 16 one at three delays (one of
    them with bfloat16 gradients), every element of every array:
    the binary32 oracle runs on all host threads (one contiguous element range
    each -- the rules are element-wise) through warm-up, the first local
    update, a Pull and the refresh after it, and the whole GPU state is
    compared bit for bit at two points of the schedule."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    import psutil
    from paper_2012_05396_amd import binding as B
    # a box too small for this test fails it: a skip would hide the coverage
    assert psutil.virtual_memory().available >= 64 * 2 ** 30, \
        "needs 64 GB of free host memory for the oracle's copy of the model"
    wl = workloads.workload(name)
    dev = torch.device("cuda", 0)
    numel = workloads.numels(wl.tensors)
    N, K, k, W = sum(numel), wl.K, wl.k, wl.W
    print("case: %s every element, N=%d K=%d k=%d grad_dtype=%d" % (name, N, K, k, gd), flush=True)
    wflat, offs = workloads.initial_weights(wl, device=dev)
    weights = workloads.views(wflat, wl.tensors, offs)
    P = 2
    gsets = [workloads.gradient_set(wl, p, device=dev, dtype=B.GRAD_TORCH_DTYPE[gd]) for p in range(P)]
    gviews = [[workloads.views(g, wl.tensors, offs) for g in gs] for gs in gsets]
    tables = [B.GradTable(g) for g in gviews]
    host = lambda views: torch.cat([v.reshape(-1) for v in views]).to(torch.float32).cpu().numpy()
    w0 = host(weights)
    gh = [[host(v) for v in gs] for gs in gviews]
    ctx = B.Context(B.make_config(numel, K, k, W, wl.lr, wl.momentum, wl.wd,
                                  stream=torch.cuda.current_stream().cuda_stream, grad_dtype=gd), weights)
    C = min(16, len(os.sched_getaffinity(0)))
    cuts = [N * j // C for j in range(C + 1)]
    parts = [Oracle(w0[a:b], K=K, k=k, W=W, lr=wl.lr, m=wl.momentum, wd=wl.wd, mode="f32")
             for a, b in zip(cuts[:-1], cuts[1:])]
    del w0

    def same(name, got, pick):
        got = got.view(np.int32)
        for j, o in enumerate(parts):
            exp = np.asarray(pick(o), np.float32).view(np.int32)
            seg = got[cuts[j]:cuts[j + 1]]
            if not np.array_equal(seg, exp):
                bad = np.nonzero(seg != exp)[0]
                raise AssertionError("%s: %d elements differ in range %d, first at element %d"
                                     % (name, bad.size, j, cuts[j] + bad[0]))

    def compare(tag):
        torch.cuda.synchronize()
        v = ctx.ssd_get_state()
        same(tag + " w", host(weights), lambda o: o.w)
        same(tag + " mom", host(ctx.state_tensors("mom")), lambda o: o.mom)
        same(tag + " pre", host(ctx.state_tensors("pre")), lambda o: o.pre[0])
        for i in range(K):
            wl_i = host(weights) if v.w_local_is_global else host(ctx.state_tensors("w_local", i))
            same(tag + " w_local[%d]" % i, wl_i, lambda o: o.wl[i])
            if v.w_loc_where == B.SSD_W_LOC_IN_W_LOCAL:
                same(tag + " w_loc[%d]" % i, host(ctx.state_tensors("w_local", i)), lambda o: o.wloc[i])

    with ThreadPoolExecutor(C) as ex:
        for it in range(W + k + 2):
            p = it % P
            ctx.ssd_step(tables[p])
            list(ex.map(lambda j: parts[j].step([g[cuts[j]:cuts[j + 1]] for g in gh[p]]), range(C)))
            print("  iteration %d done" % it, flush=True)
            if it == W + k - 1:      # a Pull iteration: w' recorded as the global weight, w_loc in the w' arrays
                compare("after the Pull (it=%d)" % it)
            if it == W + k + 1:      # refresh-from-global, then a plain iteration
                compare("after the refresh (it=%d)" % it)
    ctx.close()
    del parts, gh, gsets, gviews, tables, wflat
    torch.cuda.empty_cache()


def test_long_schedule_stays_bit_exact():
    """300 steps-delay iterations (75 Pulls) on the ResNet-56-shaped set: no
    drift between the library and the binary32 oracle.  Against the binary64
    oracle the per-tensor error stays within 1e-5; the per-element bound is
    relaxed to 5e-5 here: the binary32 rounding errors of six times as many
    iterations as the longest configured schedule add up like a random walk
    (measured 1.1e-5 after 300 iterations)."""
    wl = workloads.workload("resnet56")._replace(steps=300)
    run_full("resnet56-long", wl=wl, tol_elem=5e-5)


def test_tensor_larger_than_2_to_31_elements():
    """64-bit offsets: one tensor of 2^31 + 1029 elements (8.6 GB per array),
    sampled at its ends, around block boundaries and at random positions,
    plus a small second tensor behind it in the arena."""
    big = 2 ** 31 + 1029
    free, _ = torch.cuda.mem_get_info()
    assert free >= 80 * 2 ** 30, "needs 80 GB of free device memory (a skip would hide the 64-bit offsets)"
    tensors = [workloads.TensorSpec("big.weight", (big,), "fc", 4096),
               workloads.TensorSpec("tail.bias", (77,), "bias", 4096)]
    wl = workloads._wl("big", tensors, 1, 2, 4, seed=777)
    rng_extra = np.random.default_rng(3)
    global EXTRA_INDICES
    EXTRA_INDICES = {0: np.concatenate([np.arange(2 ** 31 - 6, 2 ** 31 + 6),
                                        np.arange(2 ** 30 - 3, 2 ** 30 + 3),
                                        rng_extra.integers(2 ** 31, big, size=512)])}
    try:
        run_full("big", wl=wl)
    finally:
        EXTRA_INDICES = {}
