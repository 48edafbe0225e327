"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the same seeded inputs.

Bars: cache slots, page indices, visibility and V pages bit-exact; bf16 outputs within
max-abs 2e-2 and relative L2 5e-3 of the oracle; fp32 outputs within 2e-5 / 1e-5.
"""
import time

import numpy as np
import pytest

import workloads as W
from oracle import cascade_oracle as orc
from tests import _harness as Hn

pytestmark = pytest.mark.gpu

BI, CA = orc.BIDIRECTIONAL, orc.BLOCK_CAUSAL


def _say(msg):
    print(msg, flush=True)


def _one_shot(w, mode, scale=None, seed=None, rows=None, heads=None, first_block=0, k_ramp=None, bounded=False):
    """Cached blocks first_block..first_block+n_cached-1, in-flight ones right after.  Returns the
    GPU result and the oracle's as lists of per-block arrays; with bounded=True also the
    per-element error bound (tests/_harness.py: attention_element_bound)."""
    q, k, v = W.draw_config(w, seed=seed, scale=scale, k_ramp=k_ramp)
    cached = list(range(first_block, first_block + w.n_cached))
    infl = list(range(first_block + w.n_cached, first_block + w.n_cached + w.n_inflight))
    pool = Hn.gpu_setup(w, k, v, cached, infl)
    out = Hn.gpu_forward(w, pool, q, infl, mode)
    if bounded:
        ref, bound = Hn.oracle_forward_bounded(w, q, k, v, cached, infl, mode, rows=rows, heads=heads)
    else:
        ref = Hn.oracle_forward(w, q, k, v, cached, infl, mode, rows=rows, heads=heads)
    L = w.block_tokens
    outs = W.split_blocks(out, L)
    if heads is not None:
        outs = [o[:, list(heads)] for o in outs]
    if rows is not None:
        outs = [o[np.asarray(r)] for o, r in zip(outs, rows)]
    return (outs, ref, bound) if bounded else (outs, ref)


def _cat(xs):
    return np.concatenate(xs)


# --------------------------------------------------------------------------- fp32 path

def test_c1_tiny_f32_full_parity():
    w = W.CONFIGS["c1_tiny_f32"]
    for mode in (BI, CA):
        outs, ref = _one_shot(w, mode)
        Hn.assert_close(np.concatenate(outs), np.concatenate(ref), "f32", f"c1 mode={mode}")


@pytest.mark.parametrize("mode", [BI, CA])
@pytest.mark.parametrize("head_dim,dims,page", [(64, (24, 20, 20), 16), (32, (12, 10, 10), 48), (128, (44, 42, 42), 100)])
def test_f32_cascade_modes(mode, head_dim, dims, page):
    w = W.small_variant(W.CONFIGS["c1_tiny_f32"], heads=3, grid_h=5, grid_w=7, head_dim=head_dim,
                        rope_dims=dims, page_tokens=page, n_cached=2, n_inflight=3, max_inflight=3,
                        window_blocks=2)
    outs, ref = _one_shot(w, mode, seed=11, first_block=4)
    Hn.assert_close(np.concatenate(outs), np.concatenate(ref), "f32", f"f32 cascade mode={mode}")
    # peaked softmax: larger logits expose indexing slips that a near-uniform softmax hides
    outs, ref = _one_shot(w, mode, seed=12, scale=2.5)
    Hn.assert_close(np.concatenate(outs), np.concatenate(ref), "f32", f"f32 peaked mode={mode}")


# --------------------------------------------------------------------------- RoPE and cache write

@pytest.mark.parametrize("name", ["c1_tiny_f32", "c3_small"])
def test_rope3d_apply_matches_oracle(name):
    import torch
    if name == "c3_small":
        w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=5, grid_h=7, grid_w=9)
    else:
        w = W.CONFIGS[name]
    from paper_2511_20426_amd.runner import CascadePool
    pool = CascadePool.for_workload(w)
    L, H, D = w.block_tokens, w.heads, w.head_dim
    n = 2 * L + 17                                     # ragged token count spanning three blocks
    rng = np.random.default_rng(5)
    x = W.store(rng.standard_normal((n, 3, H, D), dtype=np.float32), w.dtype)   # packed q/k/v rows
    first_frame = 3 * w.frames_per_block + 1
    xt = Hn.to_torch(x, w.dtype)
    view = xt[:, 1]                                    # strided [n, H, D] view, tok_stride = 3*H*D
    y = pool.rope(view, first_frame, out=torch.zeros_like(xt)[:, 1])   # same strides as the input view
    torch.cuda.synchronize()
    got = Hn.from_torch(y.contiguous(), w.dtype)
    plane = w.grid_h * w.grid_w
    idx = np.arange(n)
    pos = np.stack([first_frame + idx // plane, (idx % plane) // w.grid_w, idx % w.grid_w], axis=1)
    ref = orc.rope3d(W.to_f64(x[:, 1]), pos, w.rope_dims, w.rope_theta)
    if w.dtype == "bf16":
        # one rounding to bf16: half an ulp of the result, plus fp32 rotation error
        tol = np.abs(ref) * 2.0 ** -8 + 1e-6
    else:
        tol = np.abs(ref) * 2.0 ** -22 + 1e-6
    assert (np.abs(got - ref) <= tol).all(), float(np.abs(got - ref).max())
    # in place gives the same bits
    z = view.clone(memory_format=torch.contiguous_format)
    pool.rope(z, first_frame, out=z)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(Hn.from_torch(z, w.dtype), got)
    # and so does a strided input rotated straight into a contiguous output, and into a view
    # with head and token strides of its own (rope3d_apply_strided)
    packed = pool.rope(view, first_frame)
    assert packed.is_contiguous()
    wide = torch.zeros((n, H + 2, D + 8), dtype=xt.dtype, device=xt.device)
    pool.rope(view, first_frame, out=wide[:, 1:H + 1, :D])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(Hn.from_torch(packed, w.dtype), got)
    np.testing.assert_array_equal(Hn.from_torch(wide[:, 1:H + 1, :D].contiguous(), w.dtype), got)
    assert not wide[:, 0].any() and not wide[:, H + 1].any() and not wide[:, :, D:].any()


_WRITE_GEOMETRIES = {
    # heads, frames per block, rows, cols
    "c3_small": (3, 3, 7, 11),
    "one_column": (2, 1, 223, 1),     # a page spans 128 rows: too many angles for the kernel's trig table
    "one_row": (1, 1, 1, 300),
    "many_frames": (2, 5, 5, 7),      # a page spans several frames
    "exact_pages": (1, 2, 8, 16),     # 256 tokens: no ragged page
}


@pytest.mark.parametrize("name", ["c1_tiny_f32"] + list(_WRITE_GEOMETRIES))
def test_cache_write_pages_bit_exact_layout(name):
    """Pool bytes after kv_cache_append: V bit-exact, rotated K within one rounding, pad rows zero,
    each page at the page-pair index the oracle's rule gives."""
    import torch
    if name in _WRITE_GEOMETRIES:
        heads, fpb, gh, gw = _WRITE_GEOMETRIES[name]
        w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=heads, frames_per_block=fpb, grid_h=gh,
                            grid_w=gw, sink_blocks=1)
    else:
        w = W.CONFIGS[name]
    from paper_2511_20426_amd.runner import CascadePool
    pool = CascadePool.for_workload(w)
    pool.pool.fill_(0xAB)                               # stale bytes must be overwritten, pads zeroed
    L, H, D, P = w.block_tokens, w.heads, w.head_dim, w.pages_per_block
    cache = orc.KVCacheOracle(w.sink_blocks, max(w.window_blocks, w.n_cached), w.max_inflight, P, H)
    rng = np.random.default_rng(9)
    for g in ((0, 4, 8) if name == "c1_tiny_f32" else (0, 3, 9)):   # three distinct slots
        k = W.store(rng.standard_normal((L, H, D), dtype=np.float32), w.dtype)
        v = W.store(rng.standard_normal((L, H, D), dtype=np.float32), w.dtype)
        slot = pool.append(g, 500, 0, Hn.to_torch(k, w.dtype), Hn.to_torch(v, w.dtype))
        assert slot == cache.append(g, 500, 0)
        torch.cuda.synchronize()
        raw = pool.pool.cpu().numpy()
        kr = orc.rope3d(W.to_f64(k), orc.token_positions(g, w.frames_per_block, w.grid_h, w.grid_w),
                        w.rope_dims, w.rope_theta)
        for h in range(H):
            for p in range(P):
                idx = cache.page_index(slot, p, h)
                assert idx == pool.ctx.kv_cache_page_index(g, p, h)
                n0 = p * w.page_tokens
                nv = min(w.page_tokens, L - n0)
                if w.dtype == "bf16":
                    Kp, Vp = Hn.decode_bf16_pages(raw, idx)
                    np.testing.assert_array_equal(Vp[:nv], v[n0:n0 + nv, h])
                    Kf = W.bf16_bits_to_f32(Kp).astype(np.float64)
                    ref = kr[n0:n0 + nv, h]
                    assert (np.abs(Kf[:nv] - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-6).all()
                    assert not Kp[nv:].any() and not Vp[nv:].any()
                else:
                    Kp, Vp = Hn.decode_f32_pages(raw, idx, w.page_tokens, D)
                    np.testing.assert_array_equal(Vp[:nv], v[n0:n0 + nv, h])
                    ref = kr[n0:n0 + nv, h]
                    assert (np.abs(Kp[:nv] - ref) <= np.abs(ref) * 2.0 ** -22 + 1e-6).all()
                    assert not Kp[nv:].any() and not Vp[nv:].any()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_append_batch_writes_the_same_pool_bytes(dtype):
    """One launch for the blocks of an iteration against one kv_cache_append per block: the
    pools must be identical byte for byte (strided K/V views out of a packed tensor)."""
    import torch
    from paper_2511_20426_amd.runner import CascadePool
    if dtype == "bf16":
        w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=5, grid_h=9, grid_w=13, sink_blocks=1)
    else:
        w = W.small_variant(W.CONFIGS["c1_tiny_f32"], heads=3, grid_h=5, grid_w=7, max_inflight=4, n_inflight=4)
    L, H, D = w.block_tokens, w.heads, w.head_dim
    one, many = CascadePool.for_workload(w), CascadePool.for_workload(w)
    rng = np.random.default_rng(17)
    ids = [2, 3, 4, 5]
    packed = [Hn.to_torch(W.store(rng.standard_normal((L, 3, H, D), dtype=np.float32), w.dtype), w.dtype)
              for _ in ids]
    # the scratch area behind the pages is not part of the comparison: clear both pools first
    one.pool.zero_(); many.pool.zero_()
    for g, x in zip(ids, packed):
        one.append(g, 250 * g, 1, x[:, 1], x[:, 2])
    slots = many.append_batch(ids, [250 * g for g in ids], 1, [x[:, 1] for x in packed], [x[:, 2] for x in packed])
    torch.cuda.synchronize()
    assert [s.astuple() for s in one.ctx.kv_cache_snapshot()] == [s.astuple() for s in many.ctx.kv_cache_snapshot()]
    assert slots == [s.slot for s in many.ctx.kv_cache_snapshot()]
    assert torch.equal(one.pool, many.pool)
    assert bool(one.pool.any())


# --------------------------------------------------------------------------- bf16 MFMA path, small shapes

SMALL = [
    # heads, grid_h, grid_w, n_cached, n_inflight     tokens/block (pages, tail)
    (3, 10, 13, 2, 3),      # 390  = 3 pages + 6
    (2, 4, 5, 1, 2),        # 60   : less than one 32-key step of a page is never full
    (1, 8, 16, 0, 5),       # 384  = exactly 3 pages, no cache at all
    (5, 13, 11, 3, 1),      # 429  : single in-flight block (cascade P1)
    (2, 19, 27, 1, 2),      # 1539 : several 256-row tiles per block + ragged rows and keys
    (1, 4, 5, 0, 1),        # 60   : the whole KV sequence is one ragged page
    (1, 8, 16, 3, 1),       # 384  : one block of queries on a cache of full pages only
]


@pytest.mark.parametrize("mode", [BI, CA])
@pytest.mark.parametrize("heads,gh,gw,nc,ni", SMALL)
def test_bf16_small_full_parity(mode, heads, gh, gw, nc, ni):
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=heads, grid_h=gh, grid_w=gw,
                        n_cached=nc, n_inflight=ni)
    _say(f"bf16 small heads={heads} grid={gh}x{gw} cached={nc} inflight={ni} mode={mode}")
    outs, ref, bound = _one_shot(w, mode, seed=21, first_block=2, bounded=True)
    Hn.assert_close(_cat(outs), _cat(ref), "bf16", "small", bound=_cat(bound))
    # Peaked softmax (inputs x4: logits x16, V x4) so that a slip on a single key shows.  The
    # bf16 rounding of rotated Q and K perturbs a logit by about 2^-9 sqrt(2/3) sigma_q sigma_k
    # = 6e-3 here (4e-4 at the nominal scale), i.e. ~0.6 % on the dominant weights, on top of
    # the ~0.3 % from rounding P and O; outputs are 4x larger.  Bars scaled accordingly.
    outs, ref, bound = _one_shot(w, mode, seed=22, scale=2.0, bounded=True)
    Hn.assert_close(_cat(outs), _cat(ref), "bf16", "small peaked", max_abs=0.12, rel=1.2e-2, bound=_cat(bound))


@pytest.mark.parametrize("mode", [BI, CA])
@pytest.mark.parametrize("heads,gh,gw,nc,infl", [(3, 10, 13, 2, (2, 3, 4)), (2, 19, 27, 1, (1, 2)), (1, 4, 5, 0, (0,)),
                                                 (2, 9, 14, 2, (2, 4, 5)), (16, 19, 27, 1, (7, 8, 9))])
def test_bf16_forward_on_unrotated_queries(mode, heads, gh, gw, nc, infl):
    """cascade_attn_forward_rope (the kernel rotates Q as it loads it) against the oracle: queries
    handed over as the strided q part of a packed projection result; ragged row tiles; in-flight
    blocks that are not consecutive in the video; a launch with split KV walks; and, as a sanity
    check, closeness to the two-launch path (rope3d_apply, then cascade_attn_forward), from which
    it differs by one rounding of Q."""
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=heads, grid_h=gh, grid_w=gw, n_cached=nc,
                        n_inflight=len(infl))
    _say(f"forward on unrotated queries: heads={heads} L={w.block_tokens} cached={nc} in flight={infl} mode={mode}")
    q, k, v = W.draw_config(w, seed=91)
    first = infl[0] - nc
    cached = list(range(first, first + nc))
    pool = Hn.gpu_setup(w, k, v, cached, list(infl))
    got = Hn.gpu_forward_rope(w, pool, q, list(infl), mode)
    ref, bound = (_cat(x) for x in Hn.oracle_forward_bounded(w, q, k, v, cached, list(infl), mode))
    Hn.assert_close(got, ref, "bf16", "forward on unrotated queries", bound=bound)
    if list(infl) == list(range(infl[0], infl[0] + len(infl))):
        two = Hn.gpu_forward(w, pool, q, list(infl), mode)
        assert Hn.rel_l2(got, two) < 3e-3
    np.testing.assert_array_equal(Hn.gpu_forward_rope(w, pool, q, list(infl), mode, packed=False), got)


def test_forward_on_unrotated_queries_rejects_what_it_does_not_cover():
    import torch
    from paper_2511_20426_amd import binding as B
    from paper_2511_20426_amd.runner import CascadePool
    w = W.CONFIGS["c1_tiny_f32"]
    q, k, v = W.draw_config(w)
    pool = Hn.gpu_setup(w, k, v, [0, 1], [2])
    x = Hn.to_torch(q, w.dtype)
    with pytest.raises(B.CascadeAttnError) as e:                     # fp32 contexts have no such kernel
        pool.forward_rope(x, [2], BI, out=torch.empty_like(x))
    assert e.value.code == B.CA_EUNSUPPORTED
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=2, grid_h=4, grid_w=5, n_cached=0, n_inflight=1)
    pool = CascadePool.for_workload(w)
    t = torch.zeros((w.block_tokens, 2, 128), dtype=torch.bfloat16, device="cuda:0")
    pool.append(2000, 0, 0, t, t)                                     # latent frames 6000..: beyond the exact range
    with pytest.raises(B.CascadeAttnError) as e:
        pool.forward_rope(t, [2000], BI, out=torch.empty_like(t))
    assert e.value.code == B.CA_EUNSUPPORTED
    with pytest.raises(B.CascadeAttnError) as e:                     # head stride shorter than a head
        pool.ctx.cascade_attn_forward_rope(t.data_ptr(), 256, 64, [2000], BI, t.data_ptr())
    assert e.value.code == B.CA_EINVAL


@pytest.mark.parametrize("mode", [BI, CA])
@pytest.mark.parametrize("ramp,bar", [((1.0, 24.0), 2e-2), ((24.0, 1.0), 2e-2), ((1.0, 400.0), 8e-2),
                                      ((1.0, 400.0, "step"), 8e-2)])
def test_bf16_moving_row_maximum(mode, ramp, bar):
    """The running exponent reference has to move: K grows (or shrinks) geometrically along the
    KV sequence, so the largest logit of a row rises by tens of log2 units over the pages (first
    case), never rises after the first page (second), or jumps by more than the fp32 exponent
    range (third, gradually; fourth, from one key to the next: exp2 of a score against a stale
    reference overflows).  Logits reach |s| ~ 25 (~ 400 in the last two cases), and the bf16
    rounding of the rotated K alone perturbs such a logit by up to |s| 2^-9 ~ 5e-2 (~ 0.8; a few
    times less in the root mean square), which the softmax turns into a relative error of that
    size on the dominant weights: the bars (relative L2 2e-2 and 8e-2, measured 6e-3 and 3e-2)
    follow from that; what the test guards is the rescaling logic, whose failures are gross (inf,
    NaN, rows off by factors)."""
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=2, grid_h=10, grid_w=13, n_cached=2, n_inflight=2)
    _say(f"bf16 moving row maximum ramp={ramp} mode={mode}")
    outs, ref, bound = _one_shot(w, mode, seed=31, k_ramp=ramp, bounded=True)
    got, want, bound = _cat(outs), _cat(ref), _cat(bound)
    assert np.isfinite(got).all()
    # The per-element bound is first order in the logit perturbation: it applies while that stays
    # well below 1 (the 24x ramps: ~5e-2); with logits of ~400 the rounding of K alone moves a
    # logit by ~1 and only the norms are compared.
    Hn.assert_close(got, want, "bf16", f"moving maximum {ramp}", max_abs=bar * float(np.abs(want).max()) * 4, rel=bar,
                    bound=bound if bar <= 2e-2 else None)


@pytest.mark.parametrize("gh,gw", [(3, 43), (3, 53), (10, 16), (7, 23), (12, 16), (223, 1), (14, 16), (15, 15),
                                   (15, 17), (16, 16)])
def test_bf16_every_ragged_tail_class(gh, gw):
    """One frame per block, so that the block length L = gh * gw can take any value: the valid
    keys of the last page (L mod 128 = 1, 31, 32, 33, 64, 95, 96, 97, 127, 0) straddle every
    32-key step boundary of the page, in both masking modes, with two blocks of queries."""
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=2, grid_h=gh, grid_w=gw, frames_per_block=1,
                        n_cached=1, n_inflight=2)
    _say(f"bf16 ragged tail class L={w.block_tokens} (mod 128 = {w.block_tokens % 128})")
    for mode in (BI, CA):
        outs, ref, bound = _one_shot(w, mode, seed=61, first_block=3, bounded=True)
        Hn.assert_close(_cat(outs), _cat(ref), "bf16", f"ragged L={w.block_tokens} mode={mode}", bound=_cat(bound))


@pytest.mark.parametrize("case", range(12))
def test_bf16_seeded_random_shapes(case):
    """Twelve seeded draws of the shape itself: heads, frames per block, grid, cache depth, blocks
    in flight, first block id and mode, each case small enough for a full comparison."""
    rng = np.random.default_rng([2024, case])
    fpb = int(rng.integers(1, 4))
    gh, gw = int(rng.integers(2, 17)), int(rng.integers(2, 21))
    nc, ni = int(rng.integers(0, 4)), int(rng.integers(1, 6))
    heads = int(rng.integers(1, 5))
    mode = BI if rng.integers(0, 2) == 0 else CA
    first = int(rng.integers(0, 6))
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=heads, grid_h=gh, grid_w=gw, frames_per_block=fpb,
                        n_cached=nc, n_inflight=ni)
    _say(f"random shape {case}: heads={heads} frames={fpb} grid={gh}x{gw} L={w.block_tokens} cached={nc} "
         f"inflight={ni} first={first} mode={mode}")
    outs, ref, bound = _one_shot(w, mode, seed=1000 + case, first_block=first, bounded=True)
    Hn.assert_close(_cat(outs), _cat(ref), "bf16", f"random shape {case}", bound=_cat(bound))


@pytest.mark.parametrize("case", range(24))
def test_bf16_seeded_random_shapes_wide(case):
    """Wider draws: up to 24 heads and 1620 tokens per block (launches with more work items than
    CUs, i.e. split KV walks and the merge kernel), with or without a sink block, nominal or
    peaked inputs, plus the forward that rotates Q itself and a random share of the same forward."""
    rng = np.random.default_rng([4242, case])
    fpb = int(rng.integers(1, 4))
    gh, gw = int(rng.integers(2, 21)), int(rng.integers(2, 28))
    nc, ni = int(rng.integers(0, 7)), int(rng.integers(1, 6))
    heads = int(rng.choice([1, 2, 3, 5, 8, 12, 16, 24]))
    mode = BI if rng.integers(0, 2) == 0 else CA
    first = int(rng.integers(0, 9))
    sink = int(rng.integers(0, 2))
    base = W.CONFIGS["c5_wan1p3b_rollout" if sink else "c3_wan1p3b_cascade5"]
    L = fpb * gh * gw
    pairs = ni * L * (nc + ni) * L * heads
    if pairs > 3e9:                           # keeps the oracle to a second or two per case
        heads = max(1, int(heads * 3e9 / pairs))
    w = W.small_variant(base, heads=heads, grid_h=gh, grid_w=gw, frames_per_block=fpb, n_cached=nc, n_inflight=ni)
    if sink and nc > 0:
        first = 0                             # the sink is block 0
    scale = float(rng.choice([0.5, 0.5, 1.0, 2.0]))
    _say(f"wide random shape {case}: heads={heads} frames={fpb} grid={gh}x{gw} L={L} cached={nc} inflight={ni} "
         f"first={first} sink={sink} mode={mode} scale={scale}")
    q, k, v = W.draw_config(w, seed=5000 + case, scale=scale)
    cached = list(range(first, first + nc))
    infl = list(range(first + nc, first + nc + ni))
    pool = Hn.gpu_setup(w, k, v, cached, infl)
    out = Hn.gpu_forward(w, pool, q, infl, mode)
    ref, bound = (_cat(x) for x in Hn.oracle_forward_bounded(w, q, k, v, cached, infl, mode))
    # logits grow with scale^2 and outputs with scale: the bars of the peaked variant, interpolated
    grow = (scale / 0.5) ** 1.3
    Hn.assert_close(out, ref, "bf16", f"wide random shape {case}", max_abs=2e-2 * grow, rel=5e-3 * grow, bound=bound)
    fused = Hn.gpu_forward_rope(w, pool, q, infl, mode, packed=bool(case % 2))
    Hn.assert_close(fused, ref, "bf16", f"wide random shape {case}, Q rotated in the kernel", max_abs=2e-2 * grow,
                    rel=5e-3 * grow, bound=bound)
    if ni > 1:
        f0 = int(rng.integers(0, ni))
        cnt = int(rng.integers(1, ni - f0 + 1))
        part = Hn.gpu_forward_share(w, pool, q, infl, mode, f0, cnt)
        Hn.assert_close(part, ref[f0 * L:(f0 + cnt) * L], "bf16", f"wide random shape {case} share ({f0},{cnt})",
                        max_abs=2e-2 * grow, rel=5e-3 * grow, bound=bound[f0 * L:(f0 + cnt) * L])


@pytest.mark.parametrize("mode", [BI, CA])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_share_of_a_forward_every_block_range(mode, dtype):
    """cascade_attn_forward_share for every range of in-flight blocks: each row against the
    oracle's result for that row in the whole cascade, and against the whole forward."""
    if dtype == "bf16":
        w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=2, grid_h=9, grid_w=13, n_cached=2, n_inflight=4)
    else:
        w = W.small_variant(W.CONFIGS["c1_tiny_f32"], heads=2, grid_h=5, grid_w=7, n_cached=1, n_inflight=4,
                            max_inflight=4)
    _say(f"share dtype={dtype} mode={mode} tokens/block={w.block_tokens}")
    q, k, v = W.draw_config(w, seed=33)
    cached = list(range(3, 3 + w.n_cached))
    infl = list(range(3 + w.n_cached, 3 + w.n_cached + w.n_inflight))
    pool = Hn.gpu_setup(w, k, v, cached, infl)
    whole = W.split_blocks(Hn.gpu_forward(w, pool, q, infl, mode), w.block_tokens)
    if dtype == "bf16":
        ref, bound = Hn.oracle_forward_bounded(w, q, k, v, cached, infl, mode)
    else:
        ref, bound = Hn.oracle_forward(w, q, k, v, cached, infl, mode), None
    for first in range(w.n_inflight):
        for count in range(1, w.n_inflight - first + 1):
            part = Hn.gpu_forward_share(w, pool, q, infl, mode, first, count)
            Hn.assert_close(part, _cat(ref[first:first + count]), dtype, f"share ({first},{count})",
                            bound=None if bound is None else _cat(bound[first:first + count]))
            same = np.concatenate(whole[first:first + count])
            if dtype == "bf16":
                keys = (w.n_cached + (first + 1 if mode == CA else w.n_inflight)) * w.block_tokens
                assert (np.abs(part - same) <= _reordering_bound(part, same, v, keys)).all()
            else:
                np.testing.assert_array_equal(part, same)     # one thread per row: tiling cannot matter


@pytest.mark.parametrize("mode", [BI, CA])
@pytest.mark.parametrize("gh,gw", [(4, 5), (6, 9)])
def test_bf16_largest_configuration(mode, gh, gw):
    """The limits of a context: 32 KV blocks (1 sink + 23 clean + 8 in flight) and 8 query
    segments in block-causal mode, on a small token grid."""
    w = W.small_variant(W.CONFIGS["c5_wan1p3b_rollout"], heads=2, grid_h=gh, grid_w=gw, window_blocks=23,
                        max_inflight=8, n_cached=24, n_inflight=8)
    _say(f"largest configuration grid={gh}x{gw} mode={mode}")
    outs, ref, bound = _one_shot(w, mode, seed=71, bounded=True)
    Hn.assert_close(_cat(outs), _cat(ref), "bf16", "32 KV blocks, 8 in flight", bound=_cat(bound))


def test_bf16_pool_beyond_4_gib():
    """Page addresses past 4 GiB: 32 slots x 3 pages x 1024 heads x 64 KB = 6.4 GB of pages, the
    blocks in the last two slots (byte offsets 6.0 and 6.2 GB), checked on the first, a middle and
    the last head; cache write, both forwards and the page index against the oracle's rule."""
    w = W.small_variant(W.CONFIGS["c5_wan1p3b_rollout"], heads=1024, grid_h=8, grid_w=12, window_blocks=23,
                        max_inflight=8, n_cached=1, n_inflight=1)
    _say(f"pool beyond 4 GiB: heads={w.heads} L={w.block_tokens}")
    heads = (0, 517, 1023)
    q, k, v = W.draw_config(w, seed=77)
    pool = Hn.gpu_setup(w, k, v, [30], [31])
    assert pool.pool.numel() > (1 << 32)
    cache = orc.KVCacheOracle(w.sink_blocks, w.window_blocks, w.max_inflight, w.pages_per_block, w.heads)
    for g in (30, 31):
        slot = cache.append(g, 0, 0)
        for h in heads:
            idx = cache.page_index(slot, w.pages_per_block - 1, h)
            assert idx == pool.ctx.kv_cache_page_index(g, w.pages_per_block - 1, h)
    assert cache.page_index(cache.slot_of(31), 0, 0) * 65536 > (1 << 32)
    ref, bound = (_cat(x) for x in Hn.oracle_forward_bounded(w, q, k, v, [30], [31], BI, heads=heads))
    for got in (Hn.gpu_forward(w, pool, q, [31], BI), Hn.gpu_forward_rope(w, pool, q, [31], BI)):
        assert np.isfinite(got).all()
        Hn.assert_close(got[:, list(heads)], ref, "bf16", "pool beyond 4 GiB", bound=bound)
    # the V page of the last head of the last slot holds that head's V, bit for bit
    import torch
    L = w.block_tokens
    idx = pool.ctx.kv_cache_page_index(31, 0, 1023)
    raw = pool.pool[idx * 65536:(idx + 1) * 65536].cpu().numpy()
    _, Vp = Hn.decode_bf16_pages(raw, 0)
    np.testing.assert_array_equal(Vp, v[L:L + 128, 1023])


def test_bf16_single_block_modes_agree_bitwise():
    """One in-flight block: both modes are the same computation (cascade P1, Fig. 7)."""
    w = W.small_variant(W.CONFIGS["c2_wan1p3b_seq"], heads=2, grid_h=9, grid_w=14, n_cached=3)
    q, k, v = W.draw_config(w, seed=31)
    pool = Hn.gpu_setup(w, k, v, [0, 1, 2], [3])
    a = Hn.gpu_forward(w, pool, q, [3], BI)
    b = Hn.gpu_forward(w, pool, q, [3], CA)
    np.testing.assert_array_equal(a, b)


def test_bf16_zero_q_gives_mean_of_visible_v():
    """Q = 0 -> uniform softmax -> O = mean of visible V; checks the visible key count per mode
    and that pad keys of the ragged last page do not leak in."""
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=2, grid_h=7, grid_w=9, n_cached=2, n_inflight=3)
    q, k, v = W.draw_config(w, seed=41)
    q[:] = 0
    v[:] = W.f32_to_bf16_bits(np.ones(v.shape, np.float32))      # V = 1 -> O = 1 exactly iff weights sum to 1
    pool = Hn.gpu_setup(w, k, v, [0, 1], [2, 3, 4])
    for mode in (BI, CA):
        out = Hn.gpu_forward(w, pool, q, [2, 3, 4], mode)
        assert np.abs(out - 1.0).max() <= 2.0 ** -8
    _, _, v2 = W.draw_config(w, seed=42)
    pool = Hn.gpu_setup(w, k, v2, [0, 1], [2, 3, 4])
    L = w.block_tokens
    vf = W.to_f64(v2)
    for mode in (BI, CA):
        out = Hn.gpu_forward(w, pool, q, [2, 3, 4], mode)
        for i in range(3):
            nb = 2 + (3 if mode == BI else i + 1)
            mean = vf[:nb * L].mean(axis=0)
            got = out[i * L:(i + 1) * L]
            assert np.abs(got - mean[None]).max() <= np.abs(mean).max() * 2.0 ** -7 + 1e-4


def test_bf16_deterministic():
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=4, grid_h=12, grid_w=15, n_cached=2, n_inflight=3)
    q, k, v = W.draw_config(w, seed=51)
    pool = Hn.gpu_setup(w, k, v, [0, 1], [2, 3, 4])
    a = Hn.gpu_forward(w, pool, q, [2, 3, 4], BI)
    b = Hn.gpu_forward(w, pool, q, [2, 3, 4], BI)
    np.testing.assert_array_equal(a, b)


def test_step_replays_from_a_hip_graph():
    """Cache write, Q rotation and attention (with split work items, i.e. the merge kernel too)
    captured into a HIP graph after one eager warm-up call: the library launches plain kernels
    on the caller's stream, allocates nothing and sets its one-time kernel attributes on the
    first call.  Every replay, with fresh inputs and eager work in between, must reproduce the
    eager result bit for bit."""
    import torch
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=16, grid_h=19, grid_w=27, n_cached=1, n_inflight=3)
    L = w.block_tokens
    q, k, v = W.draw_config(w, seed=61)
    pool = Hn.gpu_setup(w, k, v, [0], [1, 2, 3])
    qs = Hn.to_torch(q, "bf16")
    ks, vs = Hn.to_torch(k, "bf16")[3 * L:].clone(), Hn.to_torch(v, "bf16")[3 * L:].clone()
    q_rot, out = torch.empty_like(qs), torch.empty_like(qs)

    def step():
        pool.append(3, 1000, 0, ks, vs)                      # the newest block's K/V are rewritten
        pool.rope(qs, w.frames_per_block * 1, out=q_rot)
        pool.forward(q_rot, [1, 2, 3], BI, out=out)

    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    gen = torch.Generator(device="cuda:0").manual_seed(5)
    for trial in range(3):
        for t in (qs, ks, vs):
            t.copy_((torch.randn(t.shape, generator=gen, device="cuda:0") * 0.5).to(torch.bfloat16))
        step()
        torch.cuda.synchronize()
        expect = out.clone()
        out.zero_()
        q_rot.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), expect.view(torch.int16)), f"replay {trial}"
        assert bool(out.float().abs().max() > 0)


def test_layer_in_three_launches_replays_from_a_hip_graph():
    """The three-launch layer (projection publishing K/V, attention rotating Q, output projection)
    captured into a HIP graph after one eager call: replays with fresh activations, eager work in
    between, must reproduce the eager result bit for bit (the library's device calls are kernel
    launches only, and its one-time kernel attributes are set by the eager call)."""
    import torch
    from paper_2511_20426_amd.runner import CascadePool, linear
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=4, grid_h=12, grid_w=15, n_cached=1, n_inflight=2)
    L, H, D = w.block_tokens, w.heads, w.head_dim
    width = H * D
    x_all, w_qkv = W.draw_linear(3 * L, 3 * width, width, seed=71)
    _, w_out = W.draw_linear(1, width, width, seed=72)
    pool = CascadePool.for_workload(w)
    xt, wq, wo = (Hn.to_torch(a, "bf16") for a in (x_all, w_qkv, w_out))
    q0 = pool.qkv_publish(xt[:L], wq, [0], [0], 0)                 # block 0 becomes the clean cache
    pool.ctx.kv_cache_promote(0)
    x = xt[L:].clone()
    q = torch.empty((2 * L, H, D), dtype=torch.bfloat16, device="cuda:0")
    o = torch.empty_like(q)
    y = torch.empty((2 * L, width), dtype=torch.bfloat16, device="cuda:0")

    def layer():
        pool.qkv_publish(x, wq, [1, 2], [250, 500], 0, q_out=q)     # the in-flight blocks are rewritten in place
        pool.forward_rope(q, [1, 2], BI, out=o)
        linear(o.view(2 * L, width), wo, out=y)

    layer()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer()
    gen = torch.Generator(device="cuda:0").manual_seed(9)
    for trial in range(3):
        x.copy_(torch.randn(x.shape, generator=gen, device="cuda:0").to(torch.bfloat16))
        layer()
        torch.cuda.synchronize()
        expect = y.clone()
        y.zero_(); o.zero_(); q.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), expect.view(torch.int16)), f"replay {trial}"
        assert bool(y.float().abs().max() > 0)


# --------------------------------------------------------------------------- full shapes, sampled rows

def _reordering_bound(a, b, v, keys):
    """Two GPU results of the same rows that differ only in how the KV walk was cut or tiled:
    the final bf16 rounding (2 ulps allowed) and the probabilities, which are rounded to bf16
    against another exponent reference (2^-9 relative per term, i.e. 2^-9 rms(v) / sqrt(keys) on
    the output; 8 sigma allowed)."""
    v_rms = float(np.sqrt(np.mean(W.bf16_bits_to_f32(v).astype(np.float64) ** 2)))
    return 2.0 ** -7 * np.maximum(np.abs(a), np.abs(b)) + 8 * 2.0 ** -9 * v_rms / np.sqrt(keys)


def _parity_rows(L, i, n_random, seed):
    """Rows of in-flight block i that meet the oracle at the full shapes: the first and last two
    (the last ones sit in the ragged tile: 4680 = 18 * 256 + 72), both sides of every multiple of
    128 rows -- every edge of a 256-row workgroup tile and the middle of each tile, where its
    second pair of waves starts -- in either tiling (tiles counted from the block's first row in
    a block-causal launch, from the first row of the whole batch in a bidirectional one), and
    n_random seeded rows."""
    return W.sample_rows(L, n_random, seed=seed, tile_edges=(128,), offsets=(0, (i * L) % 256))


def _full_shape(name, modes, n_random=16, shares=(), scale=None, full=False, bars=None, reorder_checks=True,
                fused=True):
    """One forward at a configuration's full shape against the oracle on every head: all rows
    (full=True) or the rows of _parity_rows; norm bars plus the per-element bound."""
    w = W.CONFIGS[name]
    t0 = time.time()
    q, k, v = W.draw_config(w, scale=scale)
    _say(f"{name}: drew inputs in {time.time() - t0:.1f}s")
    cached = list(range(w.n_cached))
    infl = list(range(w.n_cached, w.n_cached + w.n_inflight))
    pool = Hn.gpu_setup(w, k, v, cached, infl, timesteps=list(W.TIMESTEPS[::-1][:len(infl)]))
    L = w.block_tokens
    rows = None if full else [_parity_rows(L, i, n_random, seed=100 + i) for i in range(len(infl))]
    bars = bars or {}
    for mode in modes:
        t0 = time.time()
        out = Hn.gpu_forward(w, pool, q, infl, mode)
        _say(f"{name}: gpu forward mode={mode} done in {time.time() - t0:.1f}s")
        t0 = time.time()
        ref, bound = Hn.oracle_forward_bounded(w, q, k, v, cached, infl, mode, rows=rows)
        n_rows = len(infl) * L if full else sum(len(r) for r in rows)
        _say(f"{name}: oracle on {n_rows} rows x {w.heads} heads in {time.time() - t0:.1f}s")
        got = W.split_blocks(out, L) if full else [o[r] for o, r in zip(W.split_blocks(out, L), rows)]
        Hn.assert_close(_cat(got), _cat(ref), "bf16", f"{name} mode={mode}", bound=_cat(bound), **bars)
        assert np.isfinite(out).all()
        assert np.abs(out).max() <= np.abs(W.bf16_bits_to_f32(v)).max()     # convex combinations of V rows
        if reorder_checks:
            # cutting the KV walk of the last work items into page ranges (tail balancing, merged
            # afterwards) changes a result only through rounding: every element, GPU against GPU
            pool.ctx.set_kernel_variant(1)
            whole = Hn.gpu_forward(w, pool, q, infl, mode)
            pool.ctx.set_kernel_variant(0)
            gap = np.abs(out - whole)
            _say(f"{name}: split vs whole KV walks: {int((gap > 0).sum())} of {gap.size} elements differ, "
                 f"max {float(gap.max()):.2e}")
            keys = (w.n_cached + (1 if mode == CA else w.n_inflight)) * L
            bad = np.argwhere(gap > _reordering_bound(out, whole, v, keys))
            if len(bad):
                i = tuple(bad[0])
                _say(f"{name}: {len(bad)} outside the bound, first at {i}: {out[i]!r} vs {whole[i]!r}")
            assert len(bad) == 0
        if fused:
            part = Hn.gpu_forward_rope(w, pool, q, infl, mode)
            got = W.split_blocks(part, L) if full else [o[r] for o, r in zip(W.split_blocks(part, L), rows)]
            Hn.assert_close(_cat(got), _cat(ref), "bf16", f"{name} mode={mode}, Q rotated in the kernel",
                            bound=_cat(bound), **bars)
        # one device's share of the forward (queries of some in-flight blocks only): same rows,
        # tiled from the share's first row instead of the batch's
        for first, count in shares:
            part = Hn.gpu_forward_share(w, pool, q, infl, mode, first, count)
            got = [o[r] for o, r in zip(W.split_blocks(part, L), rows[first:first + count])]
            Hn.assert_close(_cat(got), _cat(ref[first:first + count]), "bf16",
                            f"{name} share ({first},{count}) mode={mode}", bound=_cat(bound[first:first + count]), **bars)
    return pool


def test_c2_wan1p3b_sequential_full_tensor():
    """Wan-1.3B shape, one block in flight on a 6-block cache: every output element (4680 rows x
    12 heads x 128) against the oracle."""
    _full_shape("c2_wan1p3b_seq", [BI], full=True)


def test_c2_wan1p3b_sequential_full_tensor_peaked():
    """The same shape with inputs x4 (logits x16, V x4): a softmax over 32760 keys that a few keys
    dominate, so that one missing or misplaced key would show.  Norm bars as for the small peaked
    cases (test_bf16_small_full_parity), per-element bound from the same error model."""
    _full_shape("c2_wan1p3b_seq", [BI], full=True, scale=2.0, bars=dict(max_abs=0.12, rel=1.2e-2),
                reorder_checks=False)


def test_c3_wan1p3b_cascade_both_modes_all_heads():
    _full_shape("c3_wan1p3b_cascade5", [BI, CA], shares=((0, 1), (3, 2)))


def test_c4_wan14b_cascade_all_heads():
    _full_shape("c4_wan14b_cascade5", [BI], shares=((2, 1),))


# --------------------------------------------------------------------------- long rollout (ring buffer)

def test_c5_rollout_ring_buffer():
    """40 cascade steps at the Wan-1.3B shape: 1 sink + 6-block window + 5 in flight, evict and
    append every step, prompt switch (re-tag) at step 20.  Slot of every append, snapshot,
    visibility and page indices are compared bit-exact with the oracle at every step; outputs are
    compared numerically, on every head and on the rows of _parity_rows, at steps that cover
    ramp-up (0, 3), the first full cascade (4), the first wrapped ring (11, block-causal), the
    steps around the prompt switch (19, 20, 21) and the end (39); at every other step on a light
    sample (four heads, four rows per block), so that every position of the ring is checked."""
    import torch
    from paper_2511_20426_amd.runner import CascadePool
    from paper_2511_20426_amd import binding as B
    w = W.CONFIGS["c5_wan1p3b_rollout"]
    L, H, D, C = w.block_tokens, w.heads, w.head_dim, w.max_inflight
    pool = CascadePool.for_workload(w)
    cache = orc.KVCacheOracle(w.sink_blocks, w.window_blocks, C, w.pages_per_block, H)
    checked = (0, 3, 4, 11, 19, 20, 21, 39)
    # which (step, position) draws the oracle will need: in-flight data of checked steps, and the
    # last write (the tc step, position 0) of every block that is cached at a checked step
    need = set()
    sim = orc.KVCacheOracle(w.sink_blocks, w.window_blocks, C, w.pages_per_block, H)
    for step in range(40):
        b, batch, _ = orc.rollout_step(sim, step, W.TIMESTEPS, 0)
        if step in checked:
            need.update((step, i) for i in range(len(batch)))
            order, states, _ = sim.kv_order([g for g, _ in batch])
            need.update((g + 4, 0) for g, st in zip(order, states) if st != orc.NOISY)
        orc.rollout_finish(sim, b, batch)
    host = {}
    final_kv = {}                                       # block -> (K, V) written at its tc step
    gen = torch.Generator(device="cuda:0")
    epoch = 0
    t_start = time.time()
    for step in range(40):
        if step == 20:
            epoch = 1
            before = pool.pool[:1 << 20].clone()
            cache.retag(epoch)
            pool.ctx.kv_cache_retag(epoch)
            assert [s.astuple() for s in pool.ctx.kv_cache_snapshot()] == cache.snapshot()
            assert torch.equal(before, pool.pool[:1 << 20])          # no K/V byte moves at a prompt switch
        b, batch = orc.cascade_schedule(step, W.TIMESTEPS, C)
        infl = [g for g, _ in batch]
        q_parts = []
        for i, (g, t) in enumerate(batch):
            if (step, i) in need:
                q, k, v = W.draw_step_block(w, step, i)
                host[(step, i)] = (q, k, v)
                qt, kt, vt = (Hn.to_torch(x, w.dtype) for x in (q, k, v))
            else:                                       # drawn on the device (seeded), bits copied back for the oracle
                gen.manual_seed(1000 * step + i)
                qt, kt, vt = ((torch.randn((L, H, D), generator=gen, device="cuda:0") * w.input_scale)
                              .to(torch.bfloat16) for _ in range(3))
                host[(step, i)] = tuple(x.view(torch.int16).cpu().numpy().view(np.uint16) for x in (qt, kt, vt))
            slot = pool.append(g, t, epoch, kt, vt)
            assert slot == cache.append(g, t, epoch)
            q_parts.append(qt)
            if t == 0:
                final_kv[g] = host[(step, i)][1:]
        assert [s.astuple() for s in pool.ctx.kv_cache_snapshot()] == cache.snapshot()
        order, states, slots = cache.kv_order(infl)
        for mode in (BI, CA):
            vis, kv_ids = pool.ctx.debug_visibility(infl, mode)
            assert kv_ids == order
            np.testing.assert_array_equal(np.array(vis, np.uint8), orc.visibility(states, order, infl, mode))
        for g, s in zip(order, slots):
            assert pool.ctx.kv_cache_page_index(g, w.pages_per_block - 1, H - 1) == \
                cache.page_index(s, w.pages_per_block - 1, H - 1)
        qcat = torch.cat(q_parts)
        qr = pool.rope(qcat, w.frames_per_block * infl[0])
        mode = BI if step != 11 else CA                 # one block-causal step on a wrapped ring
        out = pool.forward(qr, infl, mode)
        if step in checked:
            torch.cuda.synchronize()
            got = Hn.from_torch(out, w.dtype)
            kb, vb = [], []
            for g, st in zip(order, states):
                k, v = host[(step, infl.index(g))][1:] if st == orc.NOISY else final_kv[g]
                kb.append(k); vb.append(v)
            rows = [_parity_rows(L, i, 16, seed=step * 10 + i) for i in range(len(infl))]
            ref, bound = Hn.oracle_forward_bounded(w, [host[(step, i)][0] for i in range(len(infl))], None, None, None,
                                                   infl, mode, rows=rows, kv=(order, states, kb, vb))
            gsel = [got[i * L:(i + 1) * L][rows[i]] for i in range(len(infl))]
            Hn.assert_close(_cat(gsel), _cat(ref), "bf16", f"rollout step {step}", bound=_cat(bound))
            _say(f"rollout step {step}: {len(infl)} in flight, {len(order)} KV blocks, t={time.time() - t_start:.1f}s")
        else:
            # every other step: a light sample (four heads; first, last and two seeded rows of every
            # in-flight block), so that each position of the ring meets the oracle's numbers once
            torch.cuda.synchronize()
            got = Hn.from_torch(out, w.dtype)
            hs = (0, 5, 7, H - 1)
            kb, vb = [], []
            for g, st in zip(order, states):
                k, v = host[(step, infl.index(g))][1:] if st == orc.NOISY else final_kv[g]
                kb.append(k); vb.append(v)
            rows = [W.sample_rows(L, 2, seed=step * 10 + i, tile_edges=()) for i in range(len(infl))]
            ref, bound = Hn.oracle_forward_bounded(w, [host[(step, i)][0] for i in range(len(infl))], None, None, None,
                                                   infl, mode, rows=rows, heads=hs, kv=(order, states, kb, vb))
            gsel = [got[i * L:(i + 1) * L][rows[i]][:, list(hs)] for i in range(len(infl))]
            Hn.assert_close(_cat(gsel), _cat(ref), "bf16", f"rollout step {step} (light)", bound=_cat(bound))
        for key in [k_ for k_ in host if k_[0] < step]:     # older steps' tensors live on only as final_kv
            del host[key]
        for g in [g_ for g_ in final_kv if g_ not in order and g_ < infl[0]]:
            del final_kv[g]
        if batch[0][1] == 0:
            pool.ctx.kv_cache_promote(b)
            cache.promote(b)
            win = cache.clean_window()
            if len(win) > w.window_blocks:
                pool.ctx.kv_cache_evict(win[0])
                cache.evict(win[0])
        assert [s.astuple() for s in pool.ctx.kv_cache_snapshot()] == cache.snapshot()
    torch.cuda.synchronize()


@pytest.mark.gpu
@pytest.mark.parametrize("mode,lag,sink,window", [(BI, None, 1, 2), (CA, None, 1, 2), (BI, 2, 1, 2), (CA, 3, 1, 2),
                                                  (BI, 5, 1, 2), (CA, None, 2, 0), (BI, None, 0, 1)])
def test_algorithm1_rollout_driver(mode, lag, sink, window):
    """A full 13-block rollout driven by the library's scheduler (ramp-up, steady state, drain) on
    a small token grid, 1 sink block + 2-block window (also: two sinks and no window at all; no
    sink and a one-block window): every output row of every iteration
    against the oracle, which follows its own transcription of Alg. 1 (lag None) or its closed
    form of the lagged cascades (lag 2, 3, 5: three, two, one block in flight) and its own cache
    state machine."""
    import torch
    from paper_2511_20426_amd.runner import CascadePool
    from paper_2511_20426_amd.rollout import CascadeRollout
    w = W.small_variant(W.CONFIGS["c5_wan1p3b_rollout"], heads=2, grid_h=6, grid_w=9, sink_blocks=sink,
                        window_blocks=window)
    L, H = w.block_tokens, w.heads
    n_blocks = 13
    _say(f"alg1 rollout driver: L={L} heads={H} mode={mode} lag={lag} sink={sink} window={window}")
    pool = CascadePool.for_workload(w)
    host, outs = {}, {}

    def qkv_fn(g, ti, it, i):
        host[(it, i)] = W.draw_step_block(w, it, i, seed=77)
        return tuple(Hn.to_torch(x, w.dtype) for x in host[(it, i)])

    def out_fn(g, ti, o):
        outs.setdefault(len(ro.records), []).append(Hn.from_torch(o, w.dtype))

    ro = CascadeRollout(pool, n_blocks, W.TIMESTEPS, qkv_fn, out_fn, mode=mode, lag=lag)
    if lag is None:
        trace = orc.algorithm1_trace(n_blocks, 5)
        assert len(trace) == n_blocks + 4
    else:
        trace = [(batch[0][0], batch[0][1], len(batch) - 1, batch) for batch in orc.cascade_type_schedule(n_blocks, 5, lag)]
        assert len(trace) == lag * (n_blocks - 1) + 5
    cache = orc.KVCacheOracle(w.sink_blocks, w.window_blocks, w.max_inflight, w.pages_per_block, H)
    final_kv = {}
    for it, (b, tau, d, batch) in enumerate(trace):
        rec = ro.step()
        torch.cuda.synchronize()
        assert [(g, ti) for g, ti, _ in rec.batch] == batch
        for i, (g, ti) in enumerate(batch):
            cache.append(g, W.TIMESTEPS[ti], 0)
            if ti == len(W.TIMESTEPS) - 1:
                final_kv[g] = host[(it, i)][1:]
        infl = [g for g, _ in batch]
        order, states, _ = cache.kv_order(infl)
        kb, vb = [], []
        for g, st in zip(order, states):
            k, v = host[(it, infl.index(g))][1:] if st == orc.NOISY else final_kv[g]
            kb.append(k); vb.append(v)
        ref, bound = Hn.oracle_forward_bounded(w, [host[(it, i)][0] for i in range(len(infl))], None, None, None,
                                               infl, mode, kv=(order, states, kb, vb))
        got = np.concatenate(outs[it])
        Hn.assert_close(got, _cat(ref), "bf16", f"alg1 iteration {it}", bound=_cat(bound))
        evicted = orc.rollout_finish(cache, b, [(g, W.TIMESTEPS[ti]) for g, ti in batch])
        assert rec.completed == (b if tau == 4 else -1)
        assert rec.evicted == (-1 if evicted is None else evicted)
        assert [s.astuple() for s in pool.ctx.kv_cache_snapshot()] == cache.snapshot()
    assert ro.step() is None
    assert [r.emitted for r in ro.records if r.emitted >= 0] == list(range(n_blocks))


@pytest.mark.parametrize("mode", [BI, CA])
def test_algorithm1_rollout_driver_with_the_publishing_projection(mode):
    """The same 13-block rollout with the layer's QKV projection in it, in the three-launch form:
    every iteration's K/V are published by the projection's own epilogue (layer_qkv_publish) and
    the attention kernel rotates the queries.  The oracle projects in fp64 (no rounding of q, k,
    v), rotates, attends; cache snapshots are compared after every iteration, outputs to the bars
    of the layer pipeline test (q, k, v are rounded to bf16 on the GPU side: relative L2 1e-2)."""
    import torch
    from paper_2511_20426_amd.runner import CascadePool
    from paper_2511_20426_amd.rollout import CascadeRollout
    w = W.small_variant(W.CONFIGS["c5_wan1p3b_rollout"], heads=2, grid_h=6, grid_w=9, sink_blocks=1, window_blocks=2)
    L, H, D = w.block_tokens, w.heads, w.head_dim
    width, n_blocks = H * D, 13
    _say(f"alg1 rollout with the publishing projection: L={L} width={width} mode={mode}")
    _, w_qkv = W.draw_linear(1, 3 * width, width, seed=91)
    wq_t = Hn.to_torch(w_qkv, "bf16")
    pool = CascadePool.for_workload(w)
    xs, outs = {}, {}

    def publish_fn(batch, epoch):
        it = len(ro.records)
        for i in range(len(batch)):
            xs[(it, i)] = W.draw_linear(L, 3 * width, width, seed=1000 + 10 * it + i, x_scale=0.5)[0]
        x = torch.cat([Hn.to_torch(xs[(it, i)], "bf16") for i in range(len(batch))])
        return pool.qkv_publish(x, wq_t, [g for g, _, _ in batch], [t for _, _, t in batch], epoch)

    def out_fn(g, ti, o):
        outs.setdefault(len(ro.records), []).append(Hn.from_torch(o, w.dtype))

    ro = CascadeRollout(pool, n_blocks, W.TIMESTEPS, out_fn=out_fn, publish_fn=publish_fn, mode=mode)
    trace = orc.algorithm1_trace(n_blocks, 5)
    cache = orc.KVCacheOracle(w.sink_blocks, w.window_blocks, w.max_inflight, w.pages_per_block, H)
    pos = lambda g: orc.token_positions(g, w.frames_per_block, w.grid_h, w.grid_w)
    wf = W.to_f64(w_qkv)
    final_kv = {}
    for it, (b, tau, d, batch) in enumerate(trace):
        rec = ro.step()
        torch.cuda.synchronize()
        assert [(g, ti) for g, ti, _ in rec.batch] == batch
        proj = {}
        for i, (g, ti) in enumerate(batch):
            cache.append(g, W.TIMESTEPS[ti], 0)
            qkv = orc.layer_linear(W.to_f64(xs[(it, i)]), wf).reshape(L, 3, H, D)
            proj[g] = (orc.rope3d(qkv[:, 0], pos(g), w.rope_dims, w.rope_theta),
                       orc.rope3d(qkv[:, 1], pos(g), w.rope_dims, w.rope_theta), qkv[:, 2])
            if ti == len(W.TIMESTEPS) - 1:
                final_kv[g] = proj[g][1:]
        infl = [g for g, _ in batch]
        order, states, _ = cache.kv_order(infl)
        kb = [proj[g][1] if st == orc.NOISY else final_kv[g][0] for g, st in zip(order, states)]
        vb = [proj[g][2] if st == orc.NOISY else final_kv[g][1] for g, st in zip(order, states)]
        ref = _cat(orc.cascade_attention([proj[g][0] for g in infl], kb, vb, orc.visibility(states, order, infl, mode)))
        got = _cat(outs[it])
        Hn.assert_close(got, ref, "bf16", f"alg1 + projection, iteration {it}",
                        max_abs=0.05 * float(np.abs(ref).max()) + 1e-3, rel=1e-2)
        orc.rollout_finish(cache, b, [(g, W.TIMESTEPS[ti]) for g, ti in batch])
        assert [s.astuple() for s in pool.ctx.kv_cache_snapshot()] == cache.snapshot()
    assert ro.step() is None


def test_mfma_microbench_reports_a_plausible_ceiling():
    """The MFMA-only loop: below the nominal peak, above half of it, clock within the chip's range;
    zero operands switch less and must not be slower than random ones."""
    import torch
    from paper_2511_20426_amd import binding as B
    probe = torch.empty(1 << 16, dtype=torch.uint8, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    rnd = B.mfma_microbench(1, 20000, probe.data_ptr(), probe.numel(), stream)
    zer = B.mfma_microbench(0, 20000, probe.data_ptr(), probe.numel(), stream)
    _say(f"mfma only: random {rnd[0]:.0f} TFLOP/s at {rnd[1]:.2f} GHz, zeros {zer[0]:.0f} TFLOP/s at {zer[1]:.2f} GHz")
    for t, c in (rnd, zer):
        assert 1000.0 < t < 2600.0 and 1.0 < c < 2.6
    assert zer[0] > 0.95 * rnd[0]
    with pytest.raises(B.CascadeAttnError):
        B.mfma_microbench(2, 10, probe.data_ptr(), probe.numel(), stream)
    with pytest.raises(B.CascadeAttnError):
        B.mfma_microbench(1, 10, probe.data_ptr(), 8, stream)


# --------------------------------------------------------------------------- layer_linear_bf16

def _linear_check(got, x, w, rows, what):
    """bf16 result of an fp32-accumulated dot product against the fp64 oracle: one rounding to
    bf16 (half an ulp = 2^-9 relative; 2^-8 allowed) plus the accumulation error, bounded by a few
    2^-24 of sum_k |x||w| per addition level (1e-5 of that sum allowed)."""
    xf, wf = W.to_f64(x[rows]), W.to_f64(w)
    ref = orc.layer_linear(xf, wf)
    bound = np.abs(ref) * 2.0 ** -8 + 1e-5 * orc.layer_linear(np.abs(xf), np.abs(wf)) + 1e-30
    err = np.abs(got[rows].astype(np.float64) - ref)
    worst = float((err / bound).max())
    _say(f"[parity] {what}: max err/bound = {worst:.3f}, rel L2 = {Hn.rel_l2(got[rows], ref):.2e}")
    assert worst <= 1.0, what


@pytest.mark.parametrize("M,N,K,pad", [(300, 256, 128, 0), (1000, 512, 384, 8), (257, 768, 1024, 24), (1, 256, 128, 0),
                                       (300, 8, 128, 0), (517, 328, 256, 8), (40, 1000, 128, 16)])
def test_layer_linear_small_full(M, N, K, pad):
    """Every output element; M not a multiple of the 256-row tile, K of several loop trips,
    row strides larger than the row (pad) for all three matrices."""
    import torch
    from paper_2511_20426_amd.runner import linear
    x, w = W.draw_linear(M, N, K, seed=41)
    xt = torch.zeros((M, K + pad), dtype=torch.bfloat16, device="cuda:0")
    wt = torch.zeros((N, K + pad), dtype=torch.bfloat16, device="cuda:0")
    xt[:, :K] = Hn.to_torch(x, "bf16"); wt[:, :K] = Hn.to_torch(w, "bf16")
    yt = torch.full((M + 3, N + pad), 7.0, dtype=torch.bfloat16, device="cuda:0")
    _say(f"linear M={M} N={N} K={K} pad={pad}")
    linear(xt[:, :K], wt[:, :K], out=yt[:M, :N])
    torch.cuda.synchronize()
    got = Hn.from_torch(yt, "bf16")
    assert (got[M:] == 7.0).all() and (got[:, N:] == 7.0).all()          # nothing outside y is written
    _linear_check(got[:M, :N], x, w, np.arange(M), f"linear {M}x{N}x{K}")


def test_layer_linear_qkv_and_output_projection_shapes_sampled():
    """The two projections of a Wan-14B layer for five blocks in flight (23400 tokens, model
    width 5120): QKV 5120 -> 15360 and output 5120 -> 5120, checked on sampled rows x all columns."""
    import torch
    from paper_2511_20426_amd.runner import linear
    M, K = 23400, 5120
    rows = np.unique(np.concatenate([W.sample_rows(M, 24, seed=5, tile_edges=(256,))[:40], [M - 257, M - 256, M - 1]]))
    for N in (15360, 5120):
        x, w = W.draw_linear(M, N, K, seed=43)
        _say(f"linear M={M} N={N} K={K} sampled rows={len(rows)}")
        y = linear(Hn.to_torch(x, "bf16"), Hn.to_torch(w, "bf16"),
                   out=torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda:0"))
        torch.cuda.synchronize()
        got = Hn.from_torch(y, "bf16")
        assert np.isfinite(got).all()                        # every tile of the result was written
        _linear_check(got, x, w, rows, f"linear {M}x{N}x{K}")


def test_layer_linear_rejects_unsupported_shapes():
    import torch
    from paper_2511_20426_amd import binding as B
    t = torch.zeros((512, 512), dtype=torch.bfloat16, device="cuda:0")
    p = t.data_ptr()
    for args, code in (((p, p, p, 256, 204, 128, 512, 512, 512), B.CA_EUNSUPPORTED),   # n_out not a multiple of 8
                       ((p, p, p, 256, 256, 96, 512, 512, 512), B.CA_EUNSUPPORTED),    # k_in not a multiple of 128
                       ((p, p, p, 256, 256, 128, 64, 512, 512), B.CA_EINVAL),          # row stride shorter than the row
                       ((p, p, p + 2, 256, 256, 128, 512, 512, 512), B.CA_EINVAL),     # misaligned
                       ((0, p, p, 256, 256, 128, 512, 512, 512), B.CA_EINVAL),
                       ((p, p, p, -1, 256, 128, 512, 512, 512), B.CA_EINVAL)):
        with pytest.raises(B.CascadeAttnError) as e:
            B.layer_linear_bf16(*args)
        assert e.value.code == code, args
    # empty inputs are no-ops that succeed and write nothing
    t.fill_(3.0)
    B.layer_linear_bf16(p, p, p, 0, 256, 128, 512, 512, 512)
    torch.cuda.synchronize()
    assert bool((t == 3.0).all())


@pytest.mark.parametrize("heads,fpb,gh,gw,ids,k_in", [(2, 3, 6, 9, (3, 4, 5), 256), (4, 3, 19, 27, (0, 1), 512),
                                                      (2, 1, 16, 16, (7,), 128), (2, 1, 223, 1, (2, 3), 256),
                                                      (40, 3, 30, 52, (6, 7, 8, 9, 10), 5120)])
def test_qkv_publish_writes_the_same_pool_bytes(heads, fpb, gh, gw, ids, k_in):
    """layer_qkv_publish (projection with K/V published by its epilogue) against layer_linear_bf16
    followed by kv_cache_append_batch on the k and v columns: the page area of the two pools must
    be identical byte for byte, the queries identical to the q columns, the metadata the same.
    Shapes: ragged last pages and row tiles, a row tile whose second half lies past the block's
    last page (1539 = 6 * 256 + 3), a block of exactly two pages, a geometry too large for the
    kernel's trig table (223 x 1), and the Wan-14B projection of five blocks."""
    import torch
    from paper_2511_20426_amd.runner import CascadePool, linear
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=heads, frames_per_block=fpb, grid_h=gh, grid_w=gw,
                        sink_blocks=0)
    L, H, D = w.block_tokens, w.heads, w.head_dim
    n = len(ids) * L
    _say(f"qkv publish: heads={H} L={L} blocks={ids} k_in={k_in}")
    x, wq = W.draw_linear(n, 3 * H * D, k_in, seed=61)
    xt, wt = Hn.to_torch(x, "bf16"), Hn.to_torch(wq, "bf16")
    two, one = CascadePool.for_workload(w), CascadePool.for_workload(w)
    pages = two.pool.numel() - (256 * 256 * 132 * 4)        # the partial-result area behind the pages is not compared
    two.pool.fill_(0xAB); one.pool.fill_(0xAB)              # stale bytes: every page byte of the blocks must be written
    ts = [250 * (i + 1) for i in range(len(ids))]
    qkv = linear(xt, wt).view(n, 3, H, D)
    two.append_batch(list(ids), ts, 1, [qkv[i * L:(i + 1) * L, 1] for i in range(len(ids))],
                     [qkv[i * L:(i + 1) * L, 2] for i in range(len(ids))])
    q = one.qkv_publish(xt, wt, list(ids), ts, 1, q_out=torch.full((n, H, D), float("nan"), dtype=torch.bfloat16,
                                                                    device="cuda:0"))
    torch.cuda.synchronize()
    assert [s.astuple() for s in one.ctx.kv_cache_snapshot()] == [s.astuple() for s in two.ctx.kv_cache_snapshot()]
    assert torch.equal(q.view(torch.int16), qkv[:, 0].contiguous().view(torch.int16))
    assert torch.equal(one.pool[:pages], two.pool[:pages])
    assert bool((one.pool[:pages] != 0xAB).any())
    # and the k columns really are what the oracle's projection and rotation give (sampled block, head 0 and H-1)
    if n * k_in < 5e6:
        kf = orc.layer_linear(W.to_f64(x), W.to_f64(wq)).reshape(n, 3, H, D)[:, 1]
        raw = one.pool.cpu().numpy()
        for i, g in enumerate(ids):
            kr = orc.rope3d(kf[i * L:(i + 1) * L], orc.token_positions(g, fpb, gh, gw), w.rope_dims, w.rope_theta)
            for h in (0, H - 1):
                for p in (0, w.pages_per_block - 1):
                    Kp, _ = Hn.decode_bf16_pages(raw, one.ctx.kv_cache_page_index(g, p, h))
                    nv = min(128, L - 128 * p)
                    ref = kr[128 * p:128 * p + nv, h]
                    # two roundings to bf16 (projection result, rotated value) of values of order max|k|
                    assert (np.abs(W.bf16_bits_to_f32(Kp[:nv]) - ref) <= 2.0 ** -7 * np.abs(kf[i * L:(i + 1) * L, h]).max()).all()
                    assert not Kp[nv:].any()


def test_qkv_publish_rejects_what_it_does_not_cover():
    import torch
    from paper_2511_20426_amd import binding as B
    from paper_2511_20426_amd.runner import CascadePool
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=3, grid_h=4, grid_w=5)
    pool = CascadePool.for_workload(w)
    x = torch.zeros((w.block_tokens, 384), dtype=torch.bfloat16, device="cuda:0")
    wq = torch.zeros((3 * 384, 384), dtype=torch.bfloat16, device="cuda:0")
    before = [s.astuple() for s in pool.ctx.kv_cache_snapshot()]
    with pytest.raises(B.CascadeAttnError) as e:                     # an odd number of heads: a column tile would straddle q|k|v
        pool.qkv_publish(x, wq, [0], [0], 0)
    assert e.value.code == B.CA_EUNSUPPORTED
    assert [s.astuple() for s in pool.ctx.kv_cache_snapshot()] == before          # nothing was tagged
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=2, grid_h=4, grid_w=5)
    pool = CascadePool.for_workload(w)
    x = torch.zeros((w.block_tokens, 256), dtype=torch.bfloat16, device="cuda:0")
    wq = torch.zeros((768, 256), dtype=torch.bfloat16, device="cuda:0")
    pool.qkv_publish(x, wq, [0], [0], 0)
    pool.ctx.kv_cache_promote(0)
    with pytest.raises(B.CascadeAttnError) as e:                     # a clean block is not rewritten
        pool.qkv_publish(x, wq, [0], [0], 0)
    assert e.value.code == B.CA_ESTATE
    with pytest.raises(B.CascadeAttnError) as e:                     # k_in not a multiple of 128
        pool.ctx.layer_qkv_publish([1], [0], 0, x.data_ptr(), 256, wq.data_ptr(), 256, 192, x.data_ptr())
    assert e.value.code == B.CA_EUNSUPPORTED


def test_empty_rotation_is_a_no_op():
    import torch
    from paper_2511_20426_amd.runner import CascadePool
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=2, grid_h=4, grid_w=5)
    pool = CascadePool.for_workload(w)
    x = torch.full((4, w.heads, w.head_dim), 2.0, dtype=torch.bfloat16, device="cuda:0")
    pool.ctx.rope3d_apply(x.data_ptr(), x.data_ptr(), 0, 5, x.stride(0), x.stride(1))
    pool.ctx.rope3d_apply(0, 0, 0, 0, x.stride(0), x.stride(1))          # no pointers needed for nothing
    torch.cuda.synchronize()
    assert bool((x == 2.0).all())


@pytest.mark.parametrize("fused_q,publish", [(True, False), (False, False), (True, True)])
@pytest.mark.parametrize("mode", [BI, CA])
def test_attention_layer_pipeline(mode, fused_q, publish):
    """QKV projection -> K/V published + Q rotated (strided views of the projection's output; or Q
    rotated by the attention kernel; or, with publish, K/V published by the projection's own
    epilogue: three launches per layer) -> cascaded attention -> output projection, against the same chain in the oracle (fp64
    throughout).  The HIP path rounds q, k, v and the attention output to bf16 on the way, each
    2^-9 relative, so the bar is looser than for one stage: relative L2 1e-2 (measured 4.6e-3)."""
    import torch
    from paper_2511_20426_amd.runner import CascadePool, attention_layer
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=2, grid_h=6, grid_w=9, n_cached=1, n_inflight=2)
    L, H, D = w.block_tokens, w.heads, w.head_dim
    width = H * D
    _say(f"attention layer pipeline: L={L} width={width} mode={mode}")
    x_all, w_qkv = W.draw_linear(3 * L, 3 * width, width, seed=51)        # block 0 is cached, 1 and 2 in flight
    _, w_out = W.draw_linear(1, width, width, seed=52)
    pool = CascadePool.for_workload(w)
    xt, wq, wo = (Hn.to_torch(a, "bf16") for a in (x_all, w_qkv, w_out))
    kw = dict(rotate_q_in_kernel=fused_q, publish_in_projection=publish)
    attention_layer(pool, xt[:L], wq, wo, [0], [0], 0, BI, **kw)          # block 0 runs alone, becomes clean
    pool.ctx.kv_cache_promote(0)
    y = attention_layer(pool, xt[L:], wq, wo, [1, 2], [250, 500], 0, mode, **kw)
    torch.cuda.synchronize()
    got = Hn.from_torch(y, "bf16")
    qkv = orc.layer_linear(W.to_f64(x_all), W.to_f64(w_qkv)).reshape(3 * L, 3, H, D)
    pos = lambda g: orc.token_positions(g, w.frames_per_block, w.grid_h, w.grid_w)
    kb = [orc.rope3d(qkv[g * L:(g + 1) * L, 1], pos(g), w.rope_dims, w.rope_theta) for g in range(3)]
    vb = [qkv[g * L:(g + 1) * L, 2] for g in range(3)]
    qb = [orc.rope3d(qkv[g * L:(g + 1) * L, 0], pos(g), w.rope_dims, w.rope_theta) for g in (1, 2)]
    vis = orc.visibility([orc.CLEAN, orc.NOISY, orc.NOISY], [0, 1, 2], [1, 2], mode)
    o = np.concatenate(orc.cascade_attention(qb, kb, vb, vis)).reshape(2 * L, width)
    ref = orc.layer_linear(o, W.to_f64(w_out))
    Hn.assert_close(got, ref, "bf16", f"layer pipeline mode={mode}", max_abs=0.05 * float(np.abs(ref).max()) + 1e-3, rel=1e-2)
