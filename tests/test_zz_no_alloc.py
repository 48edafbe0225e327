"""cascade_attn_forward_static: the forward whose partial results go to the library's own static
device array, against cascade_attn_forward (partials in the caller's pool) on the same inputs.

Both run the same kernels with the same split of the KV walks, so the results must agree bit for
bit; and both must meet the oracle to the usual bars.  Two calls in a row, the second on a smaller
input (fewer heads, shorter blocks, another split), show that nothing left in the static area by
one call reaches the next.
"""
import numpy as np
import pytest

import workloads as W
from oracle import cascade_oracle as orc
from tests import _harness as Hn

pytestmark = pytest.mark.gpu


def _case(heads, gh, gw, n_cached, n_inflight, seed, mode):
    import torch
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=heads, grid_h=gh, grid_w=gw, n_cached=n_cached,
                        n_inflight=n_inflight)
    q, k, v = W.draw_config(w, seed=seed)
    cached = list(range(n_cached))
    infl = list(range(n_cached, n_cached + n_inflight))
    print(f"static scratch case: heads={heads} L={w.block_tokens} cached={n_cached} inflight={n_inflight} mode={mode}",
          flush=True)
    pool = Hn.gpu_setup(w, k, v, cached, infl)
    qr = pool.rope(Hn.to_torch(q, w.dtype), w.frames_per_block * infl[0])
    # the area in the pool and the result buffers start as NaN: a partial tile or a row that a
    # launch failed to write cannot pass for a result
    pool.pool[pool.pool.numel() - (1 << 20):].fill_(0xFF)
    plain = pool.forward(qr, infl, mode, out=torch.full_like(qr, float("nan")))
    static = pool.forward(qr, infl, mode, out=torch.full_like(qr, float("nan")), static_scratch=True)
    torch.cuda.synchronize()
    a, b = Hn.from_torch(plain, w.dtype), Hn.from_torch(static, w.dtype)
    assert np.isfinite(a).all() and np.isfinite(b).all()
    np.testing.assert_array_equal(a.view(np.uint32), b.view(np.uint32))
    ref, bound = (np.concatenate(x) for x in Hn.oracle_forward_bounded(w, q, k, v, cached, infl, mode))
    Hn.assert_close(b, ref, w.dtype, "static scratch forward", bound=bound)
    return pool


def test_static_scratch_forward_matches_the_pool_scratch_forward_twice_in_a_row():
    # Shapes chosen so that both calls split KV walks (more work items per XCD than its 32 CUs,
    # with a remainder), i.e. the partial-result area and the merge kernel are in use:
    #   16 heads x 19 row tiles = 304 columns, 38 per XCD: the last 6 items cut in 5 -> 240 partial tiles;
    #   20 heads x 5 tiles x 3 causal segments = 39 items per XCD: the last 7 cut in 2 -> 112 tiles.
    first = _case(heads=16, gh=19, gw=27, n_cached=1, n_inflight=3, seed=81, mode=orc.BIDIRECTIONAL)
    second = _case(heads=20, gh=17, gw=23, n_cached=1, n_inflight=3, seed=82, mode=orc.BLOCK_CAUSAL)
    del first, second


def test_static_scratch_forward_replays_from_a_hip_graph():
    """What the call is for: after one eager call on the device it records into a HIP graph as
    plain kernel launches, and every replay reproduces the eager result bit for bit."""
    import torch
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=16, grid_h=19, grid_w=27, n_cached=1, n_inflight=3)
    q, k, v = W.draw_config(w, seed=83)
    pool = Hn.gpu_setup(w, k, v, [0], [1, 2, 3])
    qr = pool.rope(Hn.to_torch(q, w.dtype), w.frames_per_block * 1)
    out = torch.empty_like(qr)
    pool.forward(qr, [1, 2, 3], orc.BIDIRECTIONAL, out=out, static_scratch=True)        # eager: one-time set-up happens here
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pool.forward(qr, [1, 2, 3], orc.BIDIRECTIONAL, out=out, static_scratch=True)
    gen = torch.Generator(device="cuda:0").manual_seed(4)
    for trial in range(3):
        qr.copy_((torch.randn(qr.shape, generator=gen, device="cuda:0") * 0.5).to(torch.bfloat16))
        expect = pool.forward(qr, [1, 2, 3], orc.BIDIRECTIONAL, out=torch.empty_like(qr))   # partials in the pool
        torch.cuda.synchronize()
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), expect.view(torch.int16)), f"replay {trial}"


def test_static_scratch_forward_fp32_context_is_the_plain_forward():
    import torch
    w = W.CONFIGS["c1_tiny_f32"]
    q, k, v = W.draw_config(w)
    pool = Hn.gpu_setup(w, k, v, [0, 1], [2])
    qr = pool.rope(Hn.to_torch(q, w.dtype), w.frames_per_block * 2)
    a = pool.forward(qr, [2], orc.BIDIRECTIONAL, out=torch.empty_like(qr))
    b = pool.forward(qr, [2], orc.BIDIRECTIONAL, out=torch.empty_like(qr), static_scratch=True)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
