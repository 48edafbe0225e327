"""CPU tests of the built library: exported symbols, and the host metadata (slot map, tags,
visibility, page index) compared bit-exact with the oracle's state machine.  No GPU work:
contexts are metadata-only (no pool), so nothing is launched.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as W
from oracle import cascade_oracle as orc
from paper_2511_20426_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    # every header under include/: the method's boundary and the measurement aids
    header = "".join(open(os.path.join(ROOT, "include", h)).read()
                     for h in sorted(os.listdir(os.path.join(ROOT, "include"))) if h.endswith(".h"))
    assert "ca_mfma_microbench" not in open(os.path.join(ROOT, "include", "cascade_attn.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(\w+)\s*\(", body)) - {"defined", "ceil"}
    declared = {d for d in declared if d.startswith(("ca_", "kv_cache_", "rope3d_", "cascade_", "layer_"))}
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def _cfg(w: W.Workload, **kw):
    d = dict(heads=w.heads, head_dim=w.head_dim, frames_per_block=w.frames_per_block, grid_h=w.grid_h,
             grid_w=w.grid_w, rope_dims=w.rope_dims, rope_theta=w.rope_theta, sink_blocks=w.sink_blocks,
             window_blocks=w.window_blocks, max_inflight=w.max_inflight, page_tokens=w.page_tokens,
             dtype=w.dtype)
    d.update(kw)
    return B.make_config(**d)


def test_pool_bytes():
    for name, w in W.CONFIGS.items():
        cfg = _cfg(w)
        eb = 2 if w.dtype == "bf16" else 4
        slots = w.sink_blocks + w.window_blocks + w.max_inflight
        expect = slots * w.pages_per_block * w.heads * 2 * w.page_tokens * w.head_dim * eb
        if w.dtype == "bf16":
            expect += 256 * 256 * 132 * 4          # scratch for partial results of split work items
        assert B.pool_bytes(cfg) == expect, name
    assert W.CONFIGS["c4_wan14b_cascade5"].pages_per_block == 37


def test_config_validation():
    w = W.CONFIGS["c3_wan1p3b_cascade5"]
    assert B.pool_bytes(_cfg(w, rope_dims=(44, 42, 40))) == 0          # split does not add up
    assert B.pool_bytes(_cfg(w, rope_dims=(45, 41, 42))) == 0          # odd split
    assert B.pool_bytes(_cfg(w, heads=0)) == 0
    assert B.pool_bytes(_cfg(w, rope_theta=0.0)) == 0
    assert B.pool_bytes(_cfg(w, max_inflight=0)) == 0
    # limits: at most 8 blocks in flight and 32 slots in all
    assert B.pool_bytes(_cfg(w, sink_blocks=1, window_blocks=23, max_inflight=8)) > 0
    assert B.pool_bytes(_cfg(w, sink_blocks=1, window_blocks=24, max_inflight=8)) == 0
    assert B.pool_bytes(_cfg(w, sink_blocks=0, window_blocks=6, max_inflight=9)) == 0
    with pytest.raises(B.CascadeAttnError) as e:
        B.Context(_cfg(w, head_dim=64, rope_dims=(24, 20, 20)))        # bf16 needs head_dim 128
    assert e.value.code == B.CA_EUNSUPPORTED
    with pytest.raises(B.CascadeAttnError) as e:
        B.Context(_cfg(w), pool_ptr=0, pool_nbytes=4096)               # pool size without a pool
    assert e.value.code == B.CA_EINVAL
    with pytest.raises(B.CascadeAttnError) as e:
        B.Context(_cfg(w), pool_ptr=4096 + 16, pool_nbytes=1 << 40)    # misaligned pool
    assert e.value.code == B.CA_EINVAL
    with pytest.raises(B.CascadeAttnError) as e:
        B.Context(_cfg(w), pool_ptr=4096, pool_nbytes=1 << 20)         # pool too small
    assert e.value.code == B.CA_EINVAL


def _snap(ctx):
    return [s.astuple() for s in ctx.kv_cache_snapshot()]


def test_rollout_metadata_matches_oracle_bit_exact():
    """The long-rollout configuration: 40 cascade steps, 1 sink + 6-block window, 5 in flight,
    prompt switch at step 20.  Slot of every append, snapshot after every phase, visibility
    matrices and KV order, page indices: all equal to the oracle's."""
    w = W.CONFIGS["c5_wan1p3b_rollout"]
    ctx = B.Context(_cfg(w))
    cache = orc.KVCacheOracle(w.sink_blocks, w.window_blocks, w.max_inflight, w.pages_per_block, w.heads)
    epoch = 0
    evictions = 0
    for step in range(40):
        if step == 20:
            epoch = 1
            cache.retag(epoch)
            ctx.kv_cache_retag(epoch)
            assert _snap(ctx) == cache.snapshot()
        b, batch = orc.cascade_schedule(step, W.TIMESTEPS, w.max_inflight)
        slots_lib = [ctx.kv_cache_append(g, t, epoch, 0, 0, 0, 0) for g, t in batch]
        slots_orc = [cache.append(g, t, epoch) for g, t in batch]
        assert slots_lib == slots_orc
        assert _snap(ctx) == cache.snapshot()
        infl = [g for g, _ in batch]
        order, states, slots = cache.kv_order(infl)
        for mode in (B.CA_BIDIRECTIONAL, B.CA_BLOCK_CAUSAL):
            vis, kv_ids = ctx.debug_visibility(infl, mode)
            assert kv_ids == order
            np.testing.assert_array_equal(np.array(vis, dtype=np.uint8),
                                          orc.visibility(states, order, infl, mode))
        for g, s in zip(order, slots):
            for page, head in ((0, 0), (w.pages_per_block - 1, w.heads - 1), (17, 5)):
                assert ctx.kv_cache_page_index(g, page, head) == cache.page_index(s, page, head)
        # a forward on a metadata-only context validates and then reports the missing pool
        with pytest.raises(B.CascadeAttnError) as e:
            ctx.cascade_attn_forward(0, infl, B.CA_BIDIRECTIONAL, 0)
        assert e.value.code == B.CA_ENOPOOL
        if batch[0][1] == 0:
            ctx.kv_cache_promote(b)
            cache.promote(b)
            win = cache.clean_window()
            if len(win) > w.window_blocks:
                ctx.kv_cache_evict(win[0])
                cache.evict(win[0])
                evictions += 1
        assert _snap(ctx) == cache.snapshot()
    assert evictions == 40 - 4 - 7          # first eviction once sink + 6 window blocks are clean
    snap = _snap(ctx)
    assert snap[0][:3] == (0, 0, B.CA_SINK)
    # ring wrapped at least three times
    assert max(s[1] for s in snap) >= 3 * (w.window_blocks + w.max_inflight)


@pytest.mark.parametrize("sink,window", [(0, 6), (2, 3), (1, 1), (3, 0), (0, 27)])
def test_rollout_metadata_other_cache_shapes(sink, window):
    """The same walk for other cache shapes: no sink, several sink blocks, a one-block window, no
    window at all (only sinks and the blocks in flight), the largest window a context takes."""
    w = W.CONFIGS["c5_wan1p3b_rollout"]
    ctx = B.Context(_cfg(w, sink_blocks=sink, window_blocks=window))
    cache = orc.KVCacheOracle(sink, window, w.max_inflight, w.pages_per_block, w.heads)
    for step in range(3 * (window + w.max_inflight) + 9):
        b, batch = orc.cascade_schedule(step, W.TIMESTEPS, w.max_inflight)
        ids, ts = [g for g, _ in batch], [t for _, t in batch]
        assert ctx.kv_cache_append_batch(ids, ts, 0, [0] * len(ids), [0] * len(ids), 0, 0) == \
            [cache.append(g, t, 0) for g, t in batch]
        order, states, slots = cache.kv_order(ids)
        for mode in (B.CA_BIDIRECTIONAL, B.CA_BLOCK_CAUSAL):
            vis, kv_ids = ctx.debug_visibility(ids, mode)
            assert kv_ids == order
            np.testing.assert_array_equal(np.array(vis, dtype=np.uint8), orc.visibility(states, order, ids, mode))
        if batch[0][1] == 0:
            ctx.kv_cache_promote(b)
            cache.promote(b)
            win = cache.clean_window()
            if len(win) > window:
                ctx.kv_cache_evict(win[0])
                cache.evict(win[0])
        assert _snap(ctx) == cache.snapshot()
    states = [s[2] for s in _snap(ctx)]
    assert states.count(B.CA_SINK) == sink and states.count(B.CA_CLEAN) == window


def test_error_paths_leave_state_unchanged():
    w = W.CONFIGS["c5_wan1p3b_rollout"]
    ctx = B.Context(_cfg(w, window_blocks=2, max_inflight=2))
    ctx.kv_cache_append(0, 1000, 0, 0, 0, 0, 0)
    ctx.kv_cache_append(1, 1000, 0, 0, 0, 0, 0)
    before = _snap(ctx)

    def fails(code, fn, *a):
        with pytest.raises(B.CascadeAttnError) as e:
            fn(*a)
        assert e.value.code == code, (e.value.code, code)
        assert _snap(ctx) == before

    fails(B.CA_ENOSPC, ctx.kv_cache_append, 5, 1000, 0, 0, 0, 0, 0)   # ring slot of 5 == slot of 1
    fails(B.CA_EINVAL, ctx.kv_cache_append, -1, 1000, 0, 0, 0, 0, 0)
    fails(B.CA_ENOENT, ctx.kv_cache_evict, 7)
    fails(B.CA_ENOENT, ctx.kv_cache_promote, 3)
    fails(B.CA_ENOENT, ctx.kv_cache_page_index, 9, 0, 0)
    fails(B.CA_EINVAL, ctx.kv_cache_page_index, 0, w.pages_per_block, 0)
    fails(B.CA_EINVAL, ctx.kv_cache_page_index, 0, 0, w.heads)
    fails(B.CA_ENOENT, ctx.debug_visibility, [0, 2], B.CA_BIDIRECTIONAL)
    fails(B.CA_EINVAL, ctx.debug_visibility, [1, 0], B.CA_BIDIRECTIONAL)     # not ascending
    fails(B.CA_EINVAL, ctx.debug_visibility, [0, 1], 7)                      # unknown mode
    fails(B.CA_EINVAL, ctx.debug_visibility, [], B.CA_BIDIRECTIONAL)
    fails(B.CA_EINVAL, ctx.debug_visibility, [0, 1, 2], B.CA_BIDIRECTIONAL)  # more than max_inflight
    fails(B.CA_ENOPOOL, ctx.rope3d_apply, 0, 0, 10, 0, 128, 128)
    # one device's share of a forward: the block range is checked before the pool is
    for first, count in ((-1, 1), (0, 0), (0, 3), (2, 1), (1, 2), (0, -1)):
        fails(B.CA_EINVAL, ctx.cascade_attn_forward_share, 0, [0, 1], first, count, B.CA_BIDIRECTIONAL, 0)
    fails(B.CA_ENOENT, ctx.cascade_attn_forward_share, 0, [0, 2], 0, 1, B.CA_BIDIRECTIONAL, 0)
    for first, count in ((0, 1), (1, 1), (0, 2)):
        fails(B.CA_ENOPOOL, ctx.cascade_attn_forward_share, 0, [0, 1], first, count, B.CA_BLOCK_CAUSAL, 0)
    # the forward's other forms check the same things in the same order, and all need a pool
    fails(B.CA_ENOENT, ctx.cascade_attn_forward_static, 0, [0, 2], B.CA_BIDIRECTIONAL, 0)
    fails(B.CA_ENOPOOL, ctx.cascade_attn_forward_static, 0, [0, 1], B.CA_BIDIRECTIONAL, 0)
    fails(B.CA_ENOENT, ctx.cascade_attn_forward_rope, 0, 128 * w.heads, 128, [0, 2], B.CA_BIDIRECTIONAL, 0)
    fails(B.CA_EINVAL, ctx.cascade_attn_forward_rope, 0, 128 * w.heads, 128, [1, 0], B.CA_BIDIRECTIONAL, 0)
    fails(B.CA_ENOPOOL, ctx.cascade_attn_forward_rope, 0, 128 * w.heads, 128, [0, 1], B.CA_BLOCK_CAUSAL, 0)
    # the publishing projection changes no tag without a pool to publish to
    fails(B.CA_ENOPOOL, ctx.layer_qkv_publish, [3], [0], 0, 0, 128, 0, 128, 128, 0)
    fails(B.CA_EINVAL, ctx.layer_qkv_publish, [], [], 0, 0, 128, 0, 128, 128, 0)
    fails(B.CA_EINVAL, ctx.set_kernel_variant, 12345)
    ctx.set_kernel_variant(1)
    ctx.set_kernel_variant(0)
    ctx.kv_cache_promote(0)
    before = _snap(ctx)
    assert before[0][2] == B.CA_SINK
    fails(B.CA_ESTATE, ctx.kv_cache_evict, 0)                # the sink stays
    fails(B.CA_ESTATE, ctx.kv_cache_promote, 0)
    fails(B.CA_ESTATE, ctx.kv_cache_append, 0, 0, 0, 0, 0, 0, 0)
    fails(B.CA_ESTATE, ctx.debug_visibility, [0], B.CA_BIDIRECTIONAL)   # a finished block is not in flight
    ctx.kv_cache_promote(1)                                  # block 1 is past the sink: CLEAN
    before = _snap(ctx)
    assert before[1][2] == B.CA_CLEAN
    fails(B.CA_ESTATE, ctx.kv_cache_append, 1, 0, 0, 0, 0, 0, 0)       # a clean block is not rewritten
    fails(B.CA_ESTATE, ctx.kv_cache_promote, 1)
    fails(B.CA_ESTATE, ctx.debug_visibility, [1], B.CA_BLOCK_CAUSAL)
    ctx.kv_cache_append(2, 500, 0, 0, 0, 0, 0)
    before = _snap(ctx)
    fails(B.CA_EINVAL, ctx.debug_visibility, [2, 2], B.CA_BIDIRECTIONAL)   # the same block twice
    # retag on an empty cache is a no-op that succeeds
    empty = B.Context(_cfg(w))
    empty.kv_cache_retag(3)
    assert _snap(empty) == []
    assert B.strerror(B.CA_ENOSPC) and B.strerror(-99) == "unknown error"


def test_null_context_is_rejected():
    assert B.lib.kv_cache_promote(None, 0) == B.CA_EINVAL
    assert B.lib.kv_cache_evict(None, 0) == B.CA_EINVAL
    assert B.lib.kv_cache_retag(None, 0) == B.CA_EINVAL
    assert B.lib.ca_destroy(None) == B.CA_EINVAL
    assert B.lib.ca_pool_bytes(None) == 0
    n = ctypes.c_int32()
    assert B.lib.kv_cache_snapshot(None, None, 0, ctypes.byref(n)) == B.CA_EINVAL


def test_scheduler_matches_algorithm1_trace_and_golden():
    """ca_sched_* against the oracle's transcription of Alg. 1 and the hand-derived fixture."""
    T = list(W.TIMESTEPS)
    for n_blocks in (5, 13, 20):
        tr = orc.algorithm1_trace(n_blocks, 5)
        s = B.Scheduler(n_blocks, 5, T)
        emitted, completed = [], []
        for b, tau, d, batch in tr:
            assert s.state()[:3] == (b, tau, d)
            assert s.batch() == [(g, ti, T[ti]) for g, ti in batch]
            e, c = s.advance()
            if e >= 0:
                emitted.append(e)
            if c >= 0:
                completed.append(c)
        assert s.batch() == []                                   # rollout over
        with pytest.raises(B.CascadeAttnError) as ex:
            s.advance()
        assert ex.value.code == B.CA_ESTATE
        assert emitted == list(range(n_blocks)) and completed == list(range(n_blocks))
        assert s.state()[3] == n_blocks + 4
    with open(os.path.join(ROOT, "tests", "golden", "alg1_batch_sizes_B13_G5.txt")) as f:
        golden = [int(x) for line in f if not line.startswith("#") for x in line.split()]
    s = B.Scheduler(13, 5, T)
    sizes = []
    while True:
        batch = s.batch()
        if not batch:
            break
        sizes.append(len(batch))
        s.advance()
    assert sizes == golden
    for bad in ((13, 3, T), (3, 5, T)):                          # G != |T|, fewer blocks than G
        with pytest.raises(B.CascadeAttnError) as ex:
            B.Scheduler(*bad)
        assert ex.value.code == B.CA_EUNSUPPORTED
    with pytest.raises(B.CascadeAttnError) as ex:
        B.Scheduler(0, 5, T)
    assert ex.value.code == B.CA_EINVAL


def test_lagged_scheduler_matches_closed_form():
    """ca_sched_create_lagged against the oracle's closed form for the cascade types (lag 5, 3, 2, 1)
    and an uneven lag; emitted / completed blocks in order; argument checks."""
    T = list(W.TIMESTEPS)
    for lag in (1, 2, 3, 4, 5):
        for n_blocks in (1, 2, 7, 13):
            ref = orc.cascade_type_schedule(n_blocks, len(T), lag)
            s = B.Scheduler(n_blocks, 0, T, lag=lag)
            emitted, completed = [], []
            for n, batch in enumerate(ref):
                assert s.batch() == [(g, ti, T[ti]) for g, ti in batch]
                b, tau, d, it = s.state()
                assert (b, tau, d, it) == (batch[0][0], batch[0][1], len(batch) - 1, n)
                e, c = s.advance()
                assert e == next((g for g, ti in batch if ti == len(T) - 2), -1)
                assert c == next((g for g, ti in batch if ti == len(T) - 1), -1)
                emitted += [e] if e >= 0 else []
                completed += [c] if c >= 0 else []
            assert s.batch() == [] and s.state()[2] == -1
            assert emitted == completed == list(range(n_blocks))
    for bad in (0, 6):
        with pytest.raises(B.CascadeAttnError) as ex:
            B.Scheduler(5, 0, T, lag=bad)
        assert ex.value.code == B.CA_EINVAL


def test_missing_library_is_an_import_error_not_a_fallback():
    """There is no CPU path: with no library to load, importing the package fails."""
    import subprocess
    import sys
    env = dict(os.environ, CASCADE_ATTN_LIB="/nonexistent/libcascade_attn.so")
    code = ("import sys; sys.path.insert(0, %r)\n"
            "try:\n    import paper_2511_20426_amd\nexcept ImportError as e:\n    print('ImportError', e); sys.exit(7)\n"
            % ROOT)
    r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 7 and "is missing" in r.stdout, (r.returncode, r.stdout, r.stderr)


def test_append_batch_is_the_sequence_of_appends_or_nothing():
    """kv_cache_append_batch on a metadata-only context: same slots and tags as one call per
    entry in order; any failing entry leaves everything as it was."""
    w = W.CONFIGS["c5_wan1p3b_rollout"]
    a, b = B.Context(_cfg(w)), B.Context(_cfg(w))
    cache = orc.KVCacheOracle(w.sink_blocks, w.window_blocks, w.max_inflight, w.pages_per_block, w.heads)
    for step in range(30):
        blk, batch, slots = orc.rollout_step(cache, step, W.TIMESTEPS, epoch=step // 7)
        ids, ts = [g for g, _ in batch], [t for _, t in batch]
        got = a.kv_cache_append_batch(ids, ts, step // 7, [0] * len(ids), [0] * len(ids), 0, 0)
        assert got == slots
        for g, t in batch:
            b.kv_cache_append(g, t, step // 7, 0, 0, 0, 0)
        assert _snap(a) == _snap(b) == cache.snapshot()
        evicted = orc.rollout_finish(cache, blk, batch)
        if batch[0][1] == 0:
            for c in (a, b):
                c.kv_cache_promote(blk)
                if evicted is not None:
                    c.kv_cache_evict(evicted)
    before = _snap(a)
    live = [s[1] for s in before if s[2] == B.CA_NOISY]
    ring = w.window_blocks + w.max_inflight

    def fails(code, ids, ts=None):
        with pytest.raises(B.CascadeAttnError) as e:
            a.kv_cache_append_batch(ids, ts or [0] * len(ids), 9, [0] * len(ids), [0] * len(ids), 0, 0)
        assert e.value.code == code, (e.value.code, code)
        assert _snap(a) == before

    fails(B.CA_EINVAL, [])
    fails(B.CA_EINVAL, [live[0], live[0]])                       # a block twice in one launch
    fails(B.CA_EINVAL, list(range(live[0], live[0] + 9)))        # more than 8 entries
    fails(B.CA_ENOSPC, [live[0], live[0] + ring])                # second entry's slot is the first's
    fails(B.CA_ESTATE, [live[-1], 0])                            # the sink block is finished
    fails(B.CA_EINVAL, [live[0], -3])
