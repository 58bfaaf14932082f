"""Property tests (hypothesis, seeded by its own database-free settings) of the
library's host-only entry points: chunk planner, schedule function and
workspace size, over random tensor lists and schedules.  No GPU."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle.ssd_oracle import Oracle
from paper_2012_05396_amd import binding as B

SET = dict(max_examples=150, deadline=None, derandomize=True)

numel_lists = st.lists(st.one_of(st.integers(1, 9), st.integers(250, 260), st.integers(1, 70000)),
                       min_size=1, max_size=12)
chunk_sizes = st.sampled_from([0, 256, 512, 1024, 4096])


@settings(**SET)
@given(numel_lists, chunk_sizes)
def test_planner_partitions_every_tensor(numel, chunk):
    chunks, used = B.ssd_plan_chunks(numel, chunk)
    assert used == (chunk or 256)
    pos = [0] * len(numel)
    last_t = 0
    for t, off, ln in chunks:
        assert t >= last_t            # tensors in order
        last_t = t
        assert off == pos[t] and off % used == 0 and 1 <= ln <= used
        assert ln == used or off + ln == numel[t]   # only a tensor's last chunk is short
        pos[t] += ln
    assert pos == list(numel)


@settings(**SET)
@given(st.integers(0, 6), st.integers(0, 7), st.integers(1, 40))
def test_schedule_function_matches_the_oracle_schedule(W, k, extra):
    """The oracle walks Algorithm 1 / 2 with its own counters; the library's
    pure function must name the same kind of iteration at every step, and its
    pre_weight action must be what Algorithm 2 does at local update d."""
    o = Oracle(np.zeros(1, np.float32), K=1, k=k, W=W, lr=0.1, m=0.9, wd=0.0)
    g = [np.zeros(1, np.float32)]
    for it in range(W + extra):
        d = o.d
        kind, pre = B.ssd_step_kind_of(it, W, k, d)
        assert kind == o.step(g)
        if kind >= B.SSD_STEP_DELAY:
            assert pre == (B.SSD_PRE_INIT if d == 0 else B.SSD_PRE_REFRESH if d % k == 0 else B.SSD_PRE_KEEP)
            assert (kind == B.SSD_STEP_DELAY_PULL) == (d % k == k - 1)
            assert o.d == d + 1
        else:
            assert pre == B.SSD_PRE_KEEP and (k == 0 or it < W)
            assert (kind == B.SSD_STEP_WARMUP_LAST) == (k > 0 and it == W - 1)


@settings(**SET)
@given(numel_lists, st.integers(1, 16), st.integers(0, 5), chunk_sizes, st.sampled_from([0, 1, 2]))
def test_workspace_holds_the_state_arrays(numel, K, k, chunk, gd):
    """At least (1 + [k > 0] * (2 + 2K)) arrays of the padded arena, 256-byte
    granular, independent of the gradient element type, monotone in K."""
    def ws(K_):
        return B.ssd_workspace_bytes(B.make_config(numel, K_, k, 1, 0.1, 0.9, 1e-4, chunk_elems=chunk,
                                                   grad_dtype=gd))
    c = chunk or 256
    arena = sum(-(-n // c) * c for n in numel)
    n = ws(K)
    arrays = 1 + ((2 + 2 * K) if k > 0 else 0)
    assert n >= arrays * arena * 4 and n % 256 == 0
    assert n == B.ssd_workspace_bytes(B.make_config(numel, K, k, 1, 0.1, 0.9, 1e-4, chunk_elems=chunk))
    if K < 16:
        assert ws(K + 1) >= n


# weight "pointers": any 4-byte aligned addresses (never dereferenced); mixes 1 KiB-, 256-, 16- and 4-byte phases
addresses = st.builds(lambda base, fine, kind: base * 1024 + (fine * [1024, 256, 16, 4][kind]) % 1024,
                      st.integers(1, 1 << 30), st.integers(0, 255), st.integers(0, 3))
big_numel_lists = st.lists(st.one_of(st.integers(1, 9), st.integers(8180, 8200), st.integers(1, 70000)),
                           min_size=1, max_size=10)


@settings(**SET)
@given(big_numel_lists, chunk_sizes, st.data())
def test_arena_follows_the_weight_pointers_and_covers_every_element_once(numel, chunk, data):
    """Large 16-byte aligned tensors sit in the arena at their weight pointer's
    phase inside a 1 KiB line (so arena tiles are aligned pieces of the caller's
    arrays); every other tensor starts its first block; tensors own disjoint
    runs of whole blocks in order; every element lies in exactly one block; the
    layout never needs more workspace than the size quoted without pointers."""
    addr = [data.draw(addresses) for _ in numel]
    cfg = B.make_config(numel, 3, 2, 1, 0.1, 0.9, 1e-4, chunk_elems=chunk)
    off, blocks, nbytes = B.ssd_plan_arena(cfg, addr)
    c = chunk or 256
    assert nbytes <= B.ssd_workspace_bytes(cfg)
    end_prev = 0
    for t, n in enumerate(numel):
        lead = off[t] % c
        if n >= 32 * 256 and addr[t] % 16 == 0:
            assert lead == (addr[t] % 1024) // 4 and (addr[t] // 4 - off[t]) % 256 == 0
        else:
            assert lead == 0
        assert off[t] - lead >= end_prev and (off[t] - lead) % c == 0     # whole blocks, in order, no overlap
        end_prev = -(-(off[t] + n) // c) * c
    assert len(blocks) * c == end_prev                                     # and no gaps
    pos = [0] * len(numel)
    for b, (t, first, ln) in enumerate(blocks):
        assert first == pos[t] and 1 <= ln <= c
        assert b * c <= off[t] + first and off[t] + first + ln <= (b + 1) * c   # inside block b of the arena
        pos[t] += ln
    assert pos == list(numel)


def test_arena_without_lead_in_is_the_chunk_plan():
    numel = [5, 300, 8192, 70000]
    cfg = B.make_config(numel, 2, 2, 1, 0.1, 0.9, 1e-4)
    off, blocks, _ = B.ssd_plan_arena(cfg, [4096 * (i + 1) for i in range(4)])
    assert blocks == B.ssd_plan_chunks(numel, 0)[0]
    assert off == [0, 256, 768, 768 + 8192]
