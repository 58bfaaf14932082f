"""Shared driver of the GPU parity tests: runs the HIP library and the CPU
oracle on the same seeded inputs and compares every state array."""
import numpy as np
import torch

from oracle.ssd_oracle import Oracle
from paper_2012_05396_amd import workloads


def bits(x):
    x = x if isinstance(x, np.ndarray) else x.detach().cpu().numpy()
    return np.ascontiguousarray(x, np.float32).view(np.int32)


def cat(tensors):
    return torch.cat([t.reshape(-1) for t in tensors]).cpu().numpy()


class Model:
    """Weights and P sets of K gradient buffers for a list of tensor sizes,
    on the GPU, plus flattened host copies for the oracle.  With a 16-bit
    grad_dtype the drawn gradients are rounded to that type (torch's
    conversion) before either side sees them: the device buffers hold the
    16-bit values, the oracle gets the same values widened to float32."""

    def __init__(self, numel, K, P=3, seed=0, align=64, w_shift=0, g_shift=0, g_scale=1e-2,
                 device="cuda", grad_dtype=torch.float32):
        self.numel, self.K = list(numel), K
        rng = np.random.default_rng(seed)

        def lay(shift):
            offs, cur = [], 0
            for n in self.numel:
                cur = (cur + align - 1) // align * align
                offs.append(cur + shift)
                cur += n + shift
            return offs, cur + 4

        wo, wt = lay(w_shift)
        go, gt = lay(g_shift)
        N = sum(self.numel)
        self.w0 = rng.standard_normal(N).astype(np.float32)
        self.wflat = torch.zeros(wt, dtype=torch.float32, device=device)
        self.weights = [self.wflat[o:o + n] for o, n in zip(wo, self.numel)]
        self._scatter(self.weights, self.w0)
        self.g_host, self.g_dev, self._gflat = [], [], []
        for p in range(P):
            hs, ds = [], []
            for i in range(K):
                h = (rng.standard_normal(N) * g_scale).astype(np.float32)
                hq = torch.from_numpy(h).to(grad_dtype)
                h = hq.to(torch.float32).numpy()
                flat = torch.zeros(gt, dtype=grad_dtype, device=device)
                views = [flat[o:o + n] for o, n in zip(go, self.numel)]
                self._scatter(views, hq)
                hs.append(h)
                ds.append(views)
                self._gflat.append(flat)
            self.g_host.append(hs)
            self.g_dev.append(ds)

    def _scatter(self, views, flat_host):
        if isinstance(flat_host, np.ndarray):
            flat_host = torch.from_numpy(flat_host)
        o = 0
        for v in views:
            v.copy_(flat_host[o:o + v.numel()])
            o += v.numel()


def effective_w_local(ctx, model, i):
    """w'_i: the w_local array, or the global weight when the context records
    that every w'_i equals it."""
    v = ctx.ssd_get_state()
    if v.w_local_is_global:
        return cat(model.weights)
    return cat(ctx.state_tensors("w_local", i))


def effective_w_loc(ctx, model, i):
    """What worker i's next forward/backward would use."""
    from paper_2012_05396_amd import binding as B
    v = ctx.ssd_get_state()
    if v.w_loc_where == B.SSD_W_LOC_SEPARATE:
        return cat(ctx.state_tensors("w_loc", i))
    if v.w_loc_where == B.SSD_W_LOC_IN_W_LOCAL:
        return cat(ctx.state_tensors("w_local", i))
    return cat(model.weights)


def compare_state(ctx, model, o, exact=True, tol=1e-5, where=""):
    """Compare the library's state with the oracle's.  exact: bit for bit."""
    torch.cuda.synchronize()
    v = ctx.ssd_get_state()
    K = model.K

    def chk(name, got, exp):
        got = np.asarray(got)
        if exact:
            exp32 = np.asarray(exp, np.float32)
            gb, eb = bits(got), bits(exp32)
            # NaNs carry no value: x86 and the GPU produce different default
            # NaN signs/payloads, so "both NaN" counts as equal; everything
            # else (infinities, denormals, signed zeros) is compared by bits
            both_nan = np.isnan(got) & np.isnan(exp32)
            bad = np.nonzero((gb != eb) & ~both_nan)[0]
            assert bad.size == 0, "%s %s: %d of %d elements differ, first at %d: %r vs %r" % (
                where, name, bad.size, gb.size, bad[0], got[bad[0]], exp[bad[0]])
        else:
            # per element: |a-b| / max(|b|, 0.1 * max|b| of the tensor) -- the
            # relative error of each element, with an absolute floor for the
            # elements near zero (their error is set by the rounding of the
            # O(max|b|) terms they are the difference of).  This bounds the
            # per-tensor figure max|a-b| / max|b| by the same tolerance.
            off = 0
            for t, n in enumerate(model.numel):
                a = got[off:off + n].astype(np.float64)
                b = np.asarray(exp[off:off + n], np.float64)
                floor = max(0.1 * np.max(np.abs(b)), 1e-30)
                err = np.max(np.abs(a - b) / np.maximum(np.abs(b), floor))
                worst[0] = max(worst[0], err)
                assert err <= tol, "%s %s tensor %d: per-element rel err %.3e" % (where, name, t, err)
                off += n

    worst = [0.0]
    chk("w", cat(model.weights), o.w)
    chk("mom", cat(ctx.state_tensors("mom")), o.mom)
    if o.k == 0:
        return worst[0]
    if v.has_local:
        for i in range(K):
            chk("w_local[%d]" % i, effective_w_local(ctx, model, i), o.wl[i])
        if o.d > 0:
            chk("pre", cat(ctx.state_tensors("pre")), o.pre[0])
            for i in range(1, K):
                assert np.array_equal(bits(o.pre[i]), bits(o.pre[0]))
    for i in range(K):
        chk("w_loc[%d]" % i, effective_w_loc(ctx, model, i), o.wloc[i])
    return worst[0]


def same_bits(a, b):
    return torch.equal(a.contiguous().view(torch.int32), b.contiguous().view(torch.int32))


def assert_twin_equal(ctx, weights, twin, twin_weights, where=""):
    """Two contexts that took the same steps hold the same bits (compared on the
    GPU, tensor by tensor: their arena layouts may differ)."""
    v, u = ctx.ssd_get_state(), twin.ssd_get_state()
    for f in ("iterations", "local_updates", "in_delay_stage", "has_local", "w_local_is_global", "w_loc_where"):
        assert getattr(v, f) == getattr(u, f), (where, f)
    pairs = list(zip(weights, twin_weights)) + list(zip(ctx.state_tensors("mom"), twin.state_tensors("mom")))
    if ctx.cfg.delay_k > 0 and v.has_local:
        if v.local_updates > 0:
            pairs += list(zip(ctx.state_tensors("pre"), twin.state_tensors("pre")))
        for i in range(ctx.K):
            # the w' arrays: w'_i, or -- while w' is the global weight -- the broadcast local weights
            if not v.w_local_is_global or v.w_loc_where == 1:
                pairs += list(zip(ctx.state_tensors("w_local", i), twin.state_tensors("w_local", i)))
            if v.w_loc_where == 2:
                pairs += list(zip(ctx.state_tensors("w_loc", i), twin.state_tensors("w_loc", i)))
    for n, (a, b) in enumerate(pairs):
        assert same_bits(a, b), "%s: the two cache policies differ in array %d" % (where, n)


def run_schedule(numel, K, k, W, steps, hp=None, mode="f32", chunk_elems=256, seed=0,
                 w_shift=0, g_shift=0, g_scale=1e-2, check_every=1, P=3, lr_changes=None,
                 grad_dtype=0):
    """Drive ssd_step and the oracle side by side; compare after each step.
    grad_dtype: an ssd_grad_dtype value.  Unless hp names a cache_policy, the
    compared context runs the streaming kernels (the ones large models get) and
    a twin on a copy of the weights runs the resident ones (what the library
    would choose for inputs this small); the twin must hold the same bits."""
    from paper_2012_05396_amd import binding as B
    hp = dict(lr=0.1, momentum=0.9, wd=1e-4) if hp is None else dict(hp)
    model = Model(numel, K, P=P, seed=seed, w_shift=w_shift, g_shift=g_shift, g_scale=g_scale,
                  grad_dtype=B.GRAD_TORCH_DTYPE[grad_dtype])
    both = "cache_policy" not in hp
    if both:
        hp["cache_policy"] = B.SSD_CACHE_STREAMING
    cfg = B.make_config(numel, K, k, W, device=0,
                        stream=torch.cuda.current_stream().cuda_stream,
                        chunk_elems=chunk_elems, grad_dtype=grad_dtype, **hp)
    ctx = B.Context(cfg, model.weights)
    twin = None
    if both:
        twin_flat = model.wflat.clone()
        base = model.wflat.data_ptr()
        twin_weights = [twin_flat[(w.data_ptr() - base) // 4:(w.data_ptr() - base) // 4 + w.numel()]
                        for w in model.weights]
        tcfg = B.make_config(numel, K, k, W, device=0, stream=torch.cuda.current_stream().cuda_stream,
                             chunk_elems=chunk_elems, grad_dtype=grad_dtype,
                             **dict(hp, cache_policy=B.SSD_CACHE_RESIDENT))
        twin = B.Context(tcfg, twin_weights)
        assert ctx.ssd_get_state().streaming == 1 and twin.ssd_get_state().streaming == 0
    ohp = dict(lr=hp["lr"], m=hp["momentum"], wd=hp["wd"])
    for a in ("lr_loc", "alpha", "beta", "wd_loc"):
        if a in hp:
            ohp[a] = hp[a]
    if "rescale_grad" in hp:
        ohp["rescale"] = hp["rescale_grad"]
    if hp.get("grad_sync_exact"):
        ohp["exact_w_minus"] = True
    o = Oracle(model.w0, K=K, k=k, W=W, mode=mode, **ohp)
    tables = [B.GradTable(g) for g in model.g_dev]
    exact = mode == "f32"
    for it in range(steps):
        if lr_changes and it in lr_changes:
            lr, lr_loc = lr_changes[it]
            ctx.ssd_set_lr(lr, lr_loc)
            if twin:
                twin.ssd_set_lr(lr, lr_loc)
            o.set_lr(lr, lr_loc)
        p = it % P
        kind, _ = B.ssd_step_kind_of(it, W, k, o.d)
        ctx.ssd_step(tables[p])
        if twin:
            twin.ssd_step(tables[p])
        okind = o.step(model.g_host[p])
        assert kind == okind
        if (it + 1) % check_every == 0 or it == steps - 1:
            compare_state(ctx, model, o, exact=exact, where="it=%d kind=%d" % (it, kind))
            if twin:
                assert_twin_equal(ctx, model.weights, twin, twin_weights, where="it=%d kind=%d" % (it, kind))
    ctx.close()
    if twin:
        twin.close()
    return model, o
