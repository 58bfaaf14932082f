"""Thin ctypes binding of libssd.so: same names as include/ssd.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels;
there is no CPU fallback -- without the built library, importing fails."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SSD_LIB_PATH selects another build of the same library (kernel experiments)
LIB_PATH = os.environ.get("SSD_LIB_PATH") or os.path.join(_HERE, "libssd.so")

SSD_OK, SSD_EINVAL, SSD_EALIGN, SSD_ENOMEM, SSD_EHIP, SSD_ESTATE = 0, -1, -2, -3, -4, -5
SSD_MAX_WORKERS = 16
SSD_NOALLOC_MAX_TENSORS, SSD_NOALLOC_MAX_BLOCKS = 1024, 1048576
SSD_STEP_WARMUP, SSD_STEP_WARMUP_LAST, SSD_STEP_DELAY, SSD_STEP_DELAY_PULL = 0, 1, 2, 3
SSD_PRE_KEEP, SSD_PRE_INIT, SSD_PRE_REFRESH = 0, 1, 2
SSD_W_LOC_IS_GLOBAL, SSD_W_LOC_IN_W_LOCAL, SSD_W_LOC_SEPARATE = 0, 1, 2
SSD_GRAD_F32, SSD_GRAD_BF16, SSD_GRAD_F16 = 0, 1, 2
SSD_CACHE_AUTO, SSD_CACHE_STREAMING, SSD_CACHE_RESIDENT = 0, 1, 2
GRAD_TORCH_DTYPE = {SSD_GRAD_F32: torch.float32, SSD_GRAD_BF16: torch.bfloat16,
                    SSD_GRAD_F16: torch.float16}


class ssd_config(C.Structure):
    _fields_ = [("num_workers", C.c_int32), ("delay_k", C.c_int32),
                ("warmup_iters", C.c_int32),
                ("lr", C.c_float), ("momentum", C.c_float), ("wd", C.c_float),
                ("lr_loc", C.c_float), ("alpha", C.c_float),
                ("beta", C.c_float), ("wd_loc", C.c_float),
                ("rescale_grad", C.c_float),
                ("num_tensors", C.c_int32),
                ("numel", C.POINTER(C.c_int64)),
                ("device", C.c_int32), ("stream", C.c_void_p),
                ("chunk_elems", C.c_int32), ("waves_per_cu", C.c_int32),
                ("grad_sync_exact", C.c_int32), ("grad_dtype", C.c_int32),
                ("cache_policy", C.c_int32)]


class ssd_state_view(C.Structure):
    _fields_ = [("iterations", C.c_int64), ("local_updates", C.c_int64),
                ("in_delay_stage", C.c_int32), ("has_local", C.c_int32),
                ("w_local_is_global", C.c_int32), ("w_loc_where", C.c_int32),
                ("chunk_elems", C.c_int32), ("streaming", C.c_int32),
                ("num_chunks", C.c_int64), ("arena_elems", C.c_int64),
                ("w_local_worker_stride", C.c_int64), ("w_local_block_stride", C.c_int64),
                ("tensor_offset", C.POINTER(C.c_int64)),
                ("mom", C.c_void_p), ("pre", C.c_void_p),
                ("w_local", C.c_void_p), ("w_loc", C.c_void_p)]


class ssd_chunk(C.Structure):
    _fields_ = [("tensor", C.c_int32), ("len", C.c_int32), ("offset", C.c_int64)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libssd.so is not built (%s); run `python -m paper_2012_05396_amd.build` "
            "or __graft_entry__.build()" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    P = C.POINTER
    sigs = {
        "ssd_config_defaults": (C.c_int, [P(ssd_config), C.c_int32, C.c_float, C.c_float]),
        "ssd_lds_slice_bytes": (C.c_int, [C.c_int32, C.c_int32]),
        "ssd_workspace_bytes": (C.c_int, [P(ssd_config), P(C.c_size_t)]),
        "ssd_init": (C.c_int, [P(ssd_config), P(C.c_void_p), C.c_void_p, C.c_size_t, P(C.c_void_p)]),
        "ssd_server_aggregate_update": (C.c_int, [C.c_void_p, P(C.c_void_p)]),
        "ssd_worker_glu_update": (C.c_int, [C.c_void_p, C.c_int32, P(C.c_void_p)]),
        "ssd_worker_pull": (C.c_int, [C.c_void_p, C.c_int32]),
        "ssd_step": (C.c_int, [C.c_void_p, P(C.c_void_p)]),
        "ssd_server_aggregate_update_noalloc": (C.c_int, [C.c_int32, C.c_int32, P(C.c_int64), P(C.c_void_p),
                                                          P(C.c_void_p), P(C.c_void_p), C.c_float, C.c_float,
                                                          C.c_float, C.c_float, C.c_int32, C.c_void_p]),
        "ssd_materialize": (C.c_int, [C.c_void_p]),
        "ssd_set_lr": (C.c_int, [C.c_void_p, C.c_float, C.c_float]),
        "ssd_set_stream": (C.c_int, [C.c_void_p, C.c_void_p]),
        "ssd_set_tensor_multipliers": (C.c_int, [C.c_void_p, P(C.c_float), P(C.c_float)]),
        "ssd_get_state": (C.c_int, [C.c_void_p, P(ssd_state_view)]),
        "ssd_last_error": (C.c_char_p, [C.c_void_p]),
        "ssd_destroy": (None, [C.c_void_p]),
        "ssd_probe_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]),
        "ssd_step_kind_of": (C.c_int, [C.c_int64, C.c_int32, C.c_int32, C.c_int64, P(C.c_int32)]),
        "ssd_plan_chunks": (C.c_int, [P(C.c_int64), C.c_int32, C.c_int32, P(ssd_chunk), C.c_int64,
                                      P(C.c_int64), P(C.c_int32)]),
        "ssd_plan_arena": (C.c_int, [P(ssd_config), P(C.c_void_p), P(C.c_int64), P(ssd_chunk), C.c_int64,
                                     P(C.c_int64), P(C.c_size_t)]),
    }
    for name, (res, args) in sigs.items():
        f = getattr(lib, name)
        f.restype, f.argtypes = res, args
    return lib


lib = _load()


class SsdError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("ssd error %d: %s" % (code, msg))
        self.code = code


def _check(rc, ctx=None):
    if rc != SSD_OK:
        raise SsdError(rc, (lib.ssd_last_error(ctx) or b"").decode())


# ---- host-only helpers ----------------------------------------------------
def ssd_step_kind_of(iteration, warmup_iters, delay_k, local_updates):
    pa = C.c_int32(0)
    kind = lib.ssd_step_kind_of(iteration, warmup_iters, delay_k, local_updates, C.byref(pa))
    if kind < 0:
        raise SsdError(kind, "bad argument")
    return kind, pa.value


def ssd_plan_chunks(numel, chunk_elems=0):
    T = len(numel)
    arr = (C.c_int64 * T)(*numel)
    cnt, used = C.c_int64(0), C.c_int32(0)
    _check(lib.ssd_plan_chunks(arr, T, chunk_elems, None, 0, C.byref(cnt), C.byref(used)))
    out = (ssd_chunk * cnt.value)()
    _check(lib.ssd_plan_chunks(arr, T, chunk_elems, out, cnt.value, C.byref(cnt), C.byref(used)))
    return [(c.tensor, c.offset, c.len) for c in out], used.value


def ssd_plan_arena(cfg, weight_addresses):
    """Layout of the state arrays for these weight pointers (plain integers:
    host arithmetic only).  Returns (tensor_offset, blocks, workspace bytes),
    blocks as (tensor, first element, count) per block of a launch."""
    T = cfg.num_tensors
    assert len(weight_addresses) == T
    wp = (C.c_void_p * T)(*weight_addresses)
    off = (C.c_int64 * T)()
    nb, nbytes = C.c_int64(0), C.c_size_t(0)
    _check(lib.ssd_plan_arena(C.byref(cfg), wp, off, None, 0, C.byref(nb), C.byref(nbytes)))
    out = (ssd_chunk * nb.value)()
    _check(lib.ssd_plan_arena(C.byref(cfg), wp, off, out, nb.value, None, None))
    return list(off), [(c.tensor, c.offset, c.len) for c in out], nbytes.value


def ssd_probe_copy(src, dst, stream=None):
    """Plain device copy src -> dst (float32 tensors of equal size) with the
    library's streaming loads and stores; a measurement aid."""
    assert src.is_cuda and dst.is_cuda and src.numel() == dst.numel()
    rc = lib.ssd_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel(),
                            stream if stream is not None else torch.cuda.current_stream().cuda_stream)
    if rc != SSD_OK:
        raise SsdError(rc, "ssd_probe_copy: bad size or alignment")


def ssd_config_defaults(K, lr, wd):
    """ssd_config filled by the library with the paper's settings (Sec. 4.1,
    Table 1) for K workers, global learning rate lr and weight decay wd."""
    cfg = ssd_config()
    _check(lib.ssd_config_defaults(C.byref(cfg), K, lr, wd))
    return cfg


def ssd_lds_slice_bytes(waves_per_cu, lds_bytes_per_cu):
    n = lib.ssd_lds_slice_bytes(waves_per_cu, lds_bytes_per_cu)
    if n < 0:
        raise SsdError(n, "bad argument")
    return n


def make_config(numel, K, k, W, lr, momentum, wd, lr_loc=None, alpha=None, beta=None, wd_loc=None,
                rescale_grad=None, device=0, stream=None, chunk_elems=0, waves_per_cu=0,
                grad_sync_exact=0, grad_dtype=SSD_GRAD_F32, cache_policy=0):
    """ssd_config: the library's defaults (ssd_config_defaults: loc_lr = 4*lr,
    alpha = 2, beta = 0.5, averaged gradient, wd_loc = wd), then whatever the
    caller overrides.  Returns the struct; it keeps the numel array alive."""
    T = len(numel)
    arr = (C.c_int64 * T)(*[int(n) for n in numel])
    cfg = ssd_config_defaults(K, lr, wd)
    cfg.delay_k, cfg.warmup_iters, cfg.momentum = k, W, momentum
    for name, val in (("lr_loc", lr_loc), ("alpha", alpha), ("beta", beta), ("wd_loc", wd_loc),
                      ("rescale_grad", rescale_grad)):
        if val is not None:
            setattr(cfg, name, val)
    cfg.num_tensors, cfg.numel, cfg.device, cfg.stream = T, arr, device, stream
    cfg.chunk_elems, cfg.waves_per_cu = chunk_elems, waves_per_cu
    cfg.grad_sync_exact, cfg.grad_dtype, cfg.cache_policy = grad_sync_exact, grad_dtype, cache_policy
    cfg._keep = arr
    return cfg


def ssd_server_aggregate_update_noalloc(weights, momentum, grads, lr, m, wd, rescale_grad, device=0,
                                        stream=None):
    """Marshal torch tensors into ssd_server_aggregate_update_noalloc:
    weights, momentum: lists of T float32 device tensors (updated in place);
    grads: K lists of T float32 device tensors."""
    T, K = len(weights), len(grads)
    for t in range(T):
        n = weights[t].numel()
        for x in [weights[t], momentum[t]] + [g[t] for g in grads]:
            if not (x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.numel() == n):
                raise SsdError(SSD_EINVAL, "tensor %d: contiguous float32 device tensors of equal size expected" % t)
    numel = (C.c_int64 * T)(*[w.numel() for w in weights])
    wp = (C.c_void_p * T)(*[w.data_ptr() for w in weights])
    mp = (C.c_void_p * T)(*[x.data_ptr() for x in momentum])
    table = GradTable(grads)
    _check(lib.ssd_server_aggregate_update_noalloc(
        K, T, numel, wp, mp, table.table, lr, m, wd, rescale_grad, device,
        stream if stream is not None else torch.cuda.current_stream().cuda_stream))


def ssd_workspace_bytes(cfg):
    n = C.c_size_t(0)
    _check(lib.ssd_workspace_bytes(C.byref(cfg), C.byref(n)))
    return n.value


class GradTable:
    """Marshalled [K][T] table of device pointers for one set of gradient
    tensors; build once per set and reuse (keeps the tensors alive)."""

    def __init__(self, grads):
        self.tensors = grads
        K = len(grads)
        self.rows = []
        for row in grads:
            self.rows.append((C.c_void_p * len(row))(*[t.data_ptr() for t in row]))
        self.table = (C.c_void_p * K)(*[C.cast(r, C.c_void_p).value for r in self.rows])


class Context:
    """Owner of an ssd_ctx and of the torch-allocated workspace."""

    def __init__(self, cfg, weights):
        for t in weights:
            assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
        self.cfg = cfg
        self.weights = list(weights)
        self.K, self.T = cfg.num_workers, cfg.num_tensors
        self.numel = [cfg.numel[t] for t in range(self.T)]
        nbytes = ssd_workspace_bytes(cfg)
        dev = torch.device("cuda", cfg.device)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        wp = (C.c_void_p * self.T)(*[t.data_ptr() for t in weights])
        h = C.c_void_p(None)
        _check(lib.ssd_init(C.byref(cfg), wp, C.c_void_p(self._ws_ptr), nbytes, C.byref(h)))
        self.h = h

    def close(self):
        if self.h:
            lib.ssd_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check_row(self, row):
        """The library sees raw pointers only: a buffer of the wrong element
        type or size would be read out of bounds, so refuse it here."""
        want = GRAD_TORCH_DTYPE[self.cfg.grad_dtype]
        if len(row) != self.T:
            raise SsdError(SSD_EINVAL, "%d gradient tensors given, %d expected" % (len(row), self.T))
        for t, g in enumerate(row):
            if not (g.is_cuda and g.dtype == want and g.is_contiguous() and g.numel() == self.numel[t]):
                raise SsdError(SSD_EINVAL, "gradient tensor %d must be a contiguous %s device tensor of "
                               "%d elements" % (t, want, self.numel[t]))

    def _table(self, grads):
        if isinstance(grads, GradTable):
            if getattr(grads, "_checked_for", None) is not self:
                if len(grads.tensors) != self.K:
                    raise SsdError(SSD_EINVAL, "%d workers' gradients given, %d expected"
                                   % (len(grads.tensors), self.K))
                for row in grads.tensors:
                    self._check_row(row)
                grads._checked_for = self
            return grads
        g = GradTable(grads)
        return self._table(g)

    def ssd_server_aggregate_update(self, grads):
        g = self._table(grads)
        _check(lib.ssd_server_aggregate_update(self.h, g.table), self.h)

    def ssd_worker_glu_update(self, worker, grads_i):
        self._check_row(grads_i)
        row = (C.c_void_p * len(grads_i))(*[t.data_ptr() for t in grads_i])
        _check(lib.ssd_worker_glu_update(self.h, worker, row), self.h)

    def ssd_worker_pull(self, worker):
        _check(lib.ssd_worker_pull(self.h, worker), self.h)

    def ssd_step(self, grads):
        g = self._table(grads)
        _check(lib.ssd_step(self.h, g.table), self.h)

    def ssd_materialize(self):
        _check(lib.ssd_materialize(self.h), self.h)

    def ssd_set_lr(self, lr, lr_loc):
        _check(lib.ssd_set_lr(self.h, lr, lr_loc), self.h)

    def ssd_set_tensor_multipliers(self, lr_mult=None, wd_mult=None):
        conv = lambda m: None if m is None else (C.c_float * self.T)(*[float(x) for x in m])
        _check(lib.ssd_set_tensor_multipliers(self.h, conv(lr_mult), conv(wd_mult)), self.h)

    def ssd_set_stream(self, stream):
        """stream: a torch.cuda.Stream, a raw hipStream_t value, or None."""
        raw = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
        _check(lib.ssd_set_stream(self.h, C.c_void_p(raw)), self.h)

    def ssd_get_state(self):
        v = ssd_state_view()
        _check(lib.ssd_get_state(self.h, C.byref(v)), self.h)
        return v

    # the library-owned state as torch tensors -------------------------------
    def state_array(self, which, worker=None):
        """One state array -- which in {"mom", "pre", "w_local", "w_loc"};
        per-worker arrays need `worker` -- as a flat float32 tensor indexed by
        arena element.  A view into the workspace, except for the local
        weights of more than 8 workers, whose blocks are interleaved
        (ssd_state_view.w_local_block_stride): those are gathered into a copy."""
        v = self.ssd_get_state()
        ptr = getattr(v, which)
        if ptr is None:
            raise SsdError(SSD_ESTATE, "state array %s does not exist (delay_k = 0)" % which)
        off = ptr - self.workspace.data_ptr()
        assert off >= 0 and off % 4 == 0
        A, Ce, nb = v.arena_elems, v.chunk_elems, v.num_chunks
        count = self.K if which in ("w_local", "w_loc") else 1
        i = worker if count > 1 else 0
        flat = self.workspace[off:off + 4 * A * count].view(torch.float32)
        if which == "w_local" and v.w_local_block_stride != Ce:
            blocks = flat.as_strided((nb, Ce), (v.w_local_block_stride, 1),
                                     flat.storage_offset() + i * v.w_local_worker_stride)
            return blocks.reshape(-1)
        return flat[i * A:i * A + nb * Ce]

    def state_tensors(self, which, worker=None):
        """List of T per-tensor tensors of a state array (see state_array)."""
        v = self.ssd_get_state()
        row = self.state_array(which, worker)
        return [row[v.tensor_offset[t]:v.tensor_offset[t] + self.numel[t]] for t in range(self.T)]
