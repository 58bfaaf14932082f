"""Host-side logic of the HIP library, without a GPU: the library loads and
exports every symbol the header declares, the schedule function follows
Algorithm 1 / Algorithm 2, the chunk planner covers every element once, and
argument checking rejects bad input before anything touches a device."""
import ctypes as C
import os
import re

import pytest

from paper_2012_05396_amd import binding as B
from paper_2012_05396_amd import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "ssd.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ssd_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"ssd_init", "ssd_server_aggregate_update", "ssd_worker_glu_update", "ssd_step"} <= set(names)
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), "libssd.so does not export %s" % n


def test_binding_names_match_header():
    for n in declared_functions():
        assert hasattr(B.lib, n)
        if n in ("ssd_init", "ssd_destroy", "ssd_last_error"):
            continue   # owned by Context / error handling
        assert hasattr(B, n) or hasattr(B.Context, n), n


def test_binding_constants_and_config_layout_match_header():
    """Every enumerator and error code of the header has the same value in the
    binding, and the ctypes ssd_config lists the header's fields in order."""
    src = open(os.path.join(ROOT, "include", "ssd.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    consts = dict((n, int(v)) for n, v in re.findall(r"\b(SSD_[A-Z0-9_]+)\s*=\s*(-?\d+)", src))
    consts.update((n, int(v)) for n, v in re.findall(r"#define\s+(SSD_[A-Z0-9_]+)\s+\(?(-?\d+)\)?", src))
    assert len(consts) >= 20
    for n, v in consts.items():
        assert getattr(B, n) == v, n
    body = re.search(r"typedef struct \{(.*?)\} ssd_config;", src, flags=re.S).group(1)
    fields = re.findall(r"\b(\w+)\s*;", body)
    assert fields == [f[0] for f in B.ssd_config._fields_]
    body = re.search(r"typedef struct \{((?:(?!typedef struct).)*?)\} ssd_state_view;", src, flags=re.S).group(1)
    assert re.findall(r"\b(\w+)\s*;", body) == [f[0] for f in B.ssd_state_view._fields_]


# ---- schedule (Alg. 1 warm-up loop / steps-delay loop, Alg. 2 pre_weight) ----
@pytest.mark.parametrize("wp,k", [(0, 1), (1, 2), (3, 4), (5, 3), (9, 5), (7, 8)])
def test_step_kind_follows_algorithm_1_when_aligned(wp, k):
    assert (1 + wp) % k == 0
    W = wp + 1
    d = 0
    for num in range(W + 5 * k):
        kind, pre = B.ssd_step_kind_of(num, W, k, d)
        if num < wp:
            assert (kind, pre) == (B.SSD_STEP_WARMUP, B.SSD_PRE_KEEP)
        elif num == wp:
            assert (kind, pre) == (B.SSD_STEP_WARMUP_LAST, B.SSD_PRE_KEEP)
        else:
            # Alg. 1: Pull when num % k == k-1;  Alg. 2 with loc_update = d
            assert kind == (B.SSD_STEP_DELAY_PULL if num % k == k - 1 else B.SSD_STEP_DELAY)
            exp = B.SSD_PRE_INIT if d == 0 else (B.SSD_PRE_REFRESH if d % k == 0 else B.SSD_PRE_KEEP)
            assert pre == exp
            d += 1


def test_step_kind_matches_oracle_for_unaligned_warmup():
    import numpy as np
    from oracle.ssd_oracle import Oracle
    for W, k in [(2, 4), (0, 3), (5, 2), (1, 1), (3, 0)]:
        o = Oracle(np.zeros(1, np.float32), K=1, k=k, W=W, lr=0.1, m=0.9, wd=0.0)
        g = [np.zeros(1, np.float32)]
        for it in range(W + 3 * max(k, 1) + 1):
            kind, _ = B.ssd_step_kind_of(it, W, k, o.d)
            assert kind == o.step(g)


def test_step_kind_rejects_negative():
    with pytest.raises(B.SsdError):
        B.ssd_step_kind_of(-1, 0, 0, 0)


# ---- chunk planner -----------------------------------------------------------
@pytest.mark.parametrize("chunk", [0, 256, 1024, 8192])
@pytest.mark.parametrize("name", ["resnet20", "resnet56", "vgg16"])
def test_chunks_cover_every_element_once(name, chunk):
    numel = workloads.numels(workloads.workload(name).tensors)
    chunks, used = B.ssd_plan_chunks(numel, chunk)
    assert used % 256 == 0 and used > 0 and (chunk == used or (chunk == 0 and used == 256))
    pos = [0] * len(numel)
    for t, off, ln in chunks:          # in order, contiguous, within bounds
        assert off == pos[t] and off % used == 0 and 0 < ln <= used
        pos[t] += ln
    assert pos == numel
    assert len(chunks) == sum(-(-n // used) for n in numel)


def test_chunk_planner_edge_cases():
    assert B.ssd_plan_chunks([1], 1024) == ([(0, 0, 1)], 1024)
    assert B.ssd_plan_chunks([257], 0) == ([(0, 0, 256), (0, 256, 1)], 256)
    ch, _ = B.ssd_plan_chunks([1024, 1025], 1024)
    assert ch == [(0, 0, 1024), (1, 0, 1024), (1, 1024, 1)]
    for bad in ([0], [5, -1]):
        with pytest.raises(B.SsdError):
            B.ssd_plan_chunks(bad, 1024)
    with pytest.raises(B.SsdError):
        B.ssd_plan_chunks([10], 1000)      # not a multiple of 256


# ---- argument validation (before any device work) ------------------------------
def _cfg(**kw):
    d = dict(numel=[100, 5], K=2, k=2, W=1, lr=0.1, momentum=0.9, wd=1e-4)
    d.update(kw)
    return B.make_config(**d)


@pytest.mark.parametrize("kw", [dict(K=0), dict(K=17), dict(k=-1), dict(W=-1), dict(numel=[3, 0]),
                                dict(lr=0.0), dict(chunk_elems=100), dict(device=-1),
                                dict(waves_per_cu=-2), dict(grad_dtype=3), dict(grad_dtype=-1),
                                dict(grad_sync_exact=2), dict(cache_policy=3), dict(cache_policy=-1)])
def test_workspace_bytes_rejects_bad_config(kw):
    with pytest.raises(B.SsdError) as e:
        B.ssd_workspace_bytes(_cfg(**kw))
    assert e.value.code == B.SSD_EINVAL and len(str(e.value)) > 20


def test_model_beyond_one_launch_is_rejected():
    """A grid holds at most 2^31 - 1 blocks; 2^31 blocks of 256 elements must be
    refused by the host (before any device work), a chunk size that brings the
    count back under the limit accepted."""
    big = 256 * 2 ** 31
    with pytest.raises(B.SsdError) as e:
        B.ssd_workspace_bytes(_cfg(numel=[big]))
    assert e.value.code == B.SSD_EINVAL and "chunks" in str(e.value)
    assert B.ssd_workspace_bytes(_cfg(numel=[big], chunk_elems=512)) > 4 * big


def test_workspace_bytes_counts_the_state_arrays():
    # k = 0: momentum only.  k > 0: momentum, two pre_weight arrays, K local
    # weights, K w_loc; every tensor owns whole blocks of 256 elements.
    a = B.ssd_workspace_bytes(_cfg(k=0))
    b = B.ssd_workspace_bytes(_cfg(k=2))
    arr = (256 + 256) * 4
    assert b - a == (2 + 2 * 2) * arr


def test_init_rejects_bad_arguments_without_a_gpu():
    cfg = _cfg()
    n = B.ssd_workspace_bytes(cfg)
    h = C.c_void_p(None)
    wp = (C.c_void_p * 2)(0x1000, 0x2000)
    # NULL / misaligned workspace, NULL or misaligned weight pointers, short workspace
    assert B.lib.ssd_init(C.byref(cfg), wp, None, n, C.byref(h)) == B.SSD_EINVAL
    assert B.lib.ssd_init(C.byref(cfg), wp, C.c_void_p(0x10010), n, C.byref(h)) == B.SSD_EALIGN
    assert B.lib.ssd_init(C.byref(cfg), wp, C.c_void_p(0x10000), n - 1, C.byref(h)) == B.SSD_ENOMEM
    assert b"needed" in B.lib.ssd_last_error(None)
    bad = (C.c_void_p * 2)(0x1000, 0)
    assert B.lib.ssd_init(C.byref(cfg), bad, C.c_void_p(0x10000), n, C.byref(h)) == B.SSD_EINVAL
    bad = (C.c_void_p * 2)(0x1000, 0x2002)
    assert B.lib.ssd_init(C.byref(cfg), bad, C.c_void_p(0x10000), n, C.byref(h)) == B.SSD_EALIGN
    assert B.lib.ssd_init(C.byref(cfg), None, C.c_void_p(0x10000), n, C.byref(h)) == B.SSD_EINVAL
    assert h.value is None


def test_null_context_is_rejected():
    assert B.lib.ssd_step(None, None) == B.SSD_EINVAL
    assert B.lib.ssd_server_aggregate_update(None, None) == B.SSD_EINVAL
    assert B.lib.ssd_worker_glu_update(None, 0, None) == B.SSD_EINVAL
    assert B.lib.ssd_worker_pull(None, 0) == B.SSD_EINVAL
    assert B.lib.ssd_set_lr(None, 0.1, 0.4) == B.SSD_EINVAL
    assert B.lib.ssd_get_state(None, None) == B.SSD_EINVAL
    B.lib.ssd_destroy(None)


def test_probe_copy_validates_arguments():
    assert B.lib.ssd_probe_copy(None, None, 4, None) == B.SSD_EINVAL
    assert B.lib.ssd_probe_copy(C.c_void_p(0x1000), C.c_void_p(0x2000), 3, None) == B.SSD_EINVAL
    assert B.lib.ssd_probe_copy(C.c_void_p(0x1004), C.c_void_p(0x2000), 4, None) == B.SSD_EALIGN
    assert B.lib.ssd_probe_copy(C.c_void_p(0x1000), C.c_void_p(0x2000), 0, None) == B.SSD_OK


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "one-GPU" in (r.stderr + r.stdout)


def test_workload_shapes_match_the_published_architectures():
    exp = {"resnet20": (272474, 65), "resnet56": (855770, 173), "resnet50": (25557032, 161),
           "vgg16": (138357544, 32), "resnet152_k4": (60192808, 467),
           "alexnet": (61100840, 16), "vgg11": (132863336, 22)}
    for name, (n, t) in exp.items():
        numel = workloads.numels(workloads.workload(name).tensors)
        assert (sum(numel), len(numel)) == (n, t)


def test_multipliers_reject_null_context():
    assert B.lib.ssd_set_tensor_multipliers(None, None, None) == B.SSD_EINVAL
    assert B.lib.ssd_set_stream(None, None) == B.SSD_EINVAL
    assert B.lib.ssd_materialize(None) == B.SSD_EINVAL


# ---- occupancy cap (LDS slice per single-wave workgroup) -----------------------
@pytest.mark.parametrize("lds", [163840, 65536])
def test_lds_slice_yields_the_wave_count_it_names(lds):
    """waves * slice must fit the compute unit's LDS and one more wave must
    not: the cap means the count it names (LDS comes in 128 granules, so 13
    and 15 waves are not expressible and give 14 and 16)."""
    granule = lds // 128
    for n in range(1, 17):
        s = B.ssd_lds_slice_bytes(n, lds)
        assert s > 0 and s % granule == 0
        resident = lds // s
        assert resident == {13: 14, 15: 16}.get(n, n), (n, s, resident)
    assert B.ssd_lds_slice_bytes(0, lds) == 0 and B.ssd_lds_slice_bytes(32, lds) == 0
    for bad in [(-1, lds), (4, 0), (4, 1000)]:
        with pytest.raises(B.SsdError):
            B.ssd_lds_slice_bytes(*bad)


# ---- the paper's settings come from the library (Sec. 4.1, Table 1) -----------
def test_config_defaults_follow_the_papers_settings():
    import numpy as np
    vals = {}
    pairs = []
    for line in open(os.path.join(ROOT, "tests", "golden", "hyperparameters.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "lr":
            pairs.append((float(f[1]), float(f[3])))
        else:
            vals[f[0]] = float(f[1])
    assert len(pairs) == 2
    for lr, loc_lr in pairs:
        for K in (1, 3, 4, 16):
            c = B.ssd_config_defaults(K, lr, 1e-4)
            assert c.alpha == vals["alpha"] and c.beta == vals["beta"]
            assert c.lr_loc == np.float32(loc_lr) and c.lr == np.float32(lr)
            assert c.rescale_grad == np.float32(1.0 / K)       # Table 1: averaged gradient
            assert c.wd == np.float32(1e-4) and c.wd_loc == c.wd
            assert (c.num_workers, c.delay_k, c.warmup_iters, c.grad_dtype, c.chunk_elems) == (K, 0, 0, 0, 0)
    for badK in (0, 17):
        with pytest.raises(B.SsdError):
            B.ssd_config_defaults(badK, 0.1, 0.0)
    assert B.lib.ssd_config_defaults(None, 4, 0.1, 0.0) == B.SSD_EINVAL
    # make_config is that struct plus the caller's overrides, nothing computed in Python
    m = B.make_config([10], 4, 2, 1, 0.4, 0.9, 1e-4)
    assert (m.lr_loc, m.alpha, m.beta, m.rescale_grad) == (np.float32(1.6), 2.0, 0.5, 0.25)
    m = B.make_config([10], 4, 2, 1, 0.4, 0.9, 1e-4, lr_loc=1.0, alpha=1.0, beta=0.0, wd_loc=0.0, rescale_grad=1.0)
    assert (m.lr_loc, m.alpha, m.beta, m.wd_loc, m.rescale_grad) == (1.0, 1.0, 0.0, 0.0, 1.0)


def test_state_arrays_are_never_a_multiple_of_256_mib_apart():
    """The distance between consecutive state arrays, read off the workspace
    size (one more worker adds a w' and a w_loc array): a multiple of 64 MiB for
    large arrays, and never a multiple of 256 MiB."""
    MiB = 1 << 20
    for n, expect in ((60192808, 384 * MiB),      # 229.6 MiB -> 256 -> 384
                      (138357544, 576 * MiB),     # 527.8 MiB -> 576
                      (132863336, 640 * MiB),     # 506.8 MiB -> 512 -> 640
                      (25557032, 128 * MiB),      # 97.5 MiB -> 128
                      (198000000, 896 * MiB)):    # 755.3 MiB -> 768 -> 896
        a = B.ssd_workspace_bytes(_cfg(numel=[n], K=3, k=2))
        b = B.ssd_workspace_bytes(_cfg(numel=[n], K=4, k=2))
        # pointer tables grow by a few hundred bytes per worker
        assert 0 <= (b - a) - 2 * expect < 4096, (n, (b - a) / MiB)


def test_workspace_bound_holds_where_the_array_distance_jumps():
    """One tensor of 256 MiB - 512 B: laid out from a 1 KiB-aligned weight
    pointer its arena is exactly 256 MiB, which the library spaces 384 MiB
    apart; with a lead-in it is one block more, spaced 320 MiB.  The size
    quoted before the pointers are known must cover both."""
    n = (256 << 20) // 4 - 128
    cfg = _cfg(numel=[n], K=2, k=2)
    bound = B.ssd_workspace_bytes(cfg)
    for addr in (1 << 30, (1 << 30) + 16, (1 << 30) + 1008, (1 << 30) + 4):
        _, blocks, nbytes = B.ssd_plan_arena(cfg, [addr])
        assert nbytes <= bound, (addr, nbytes, bound)
    assert B.ssd_plan_arena(cfg, [1 << 30])[2] > B.ssd_plan_arena(cfg, [(1 << 30) + 1008])[2]
