"""Pins for the CPU oracle: brute force, closed forms, textbook special cases, invariants.

Each pin is chosen so that a plausible slip in oracle/cascade_oracle.py (a dropped
term, a wrong sign or index, a transposed operand, a mask off by one block) fails it.
None of these tests touches the GPU path.
"""
import math
import os

import numpy as np
import pytest
from scipy.special import softmax

from oracle import cascade_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


# --------------------------------------------------------------------------- brute force

def brute_force(q_raw, k_raw, v, q_blk, k_blk, q_pos, k_pos, k_is_cache, dims, theta, causal):
    """Token-by-token scalar loops, written independently of the oracle.
    q_raw[nq][H][D], k_raw[nk][H][D], v[nk][H][D]; *_blk = video block index of each token;
    *_pos = (frame,row,col) per token; k_is_cache[t] = key token belongs to a finished block."""
    nq, H, D = q_raw.shape
    nk = k_raw.shape[0]

    def rot(vec, pos):
        out = [0.0] * D
        pair = 0
        for a in range(3):
            for j in range(dims[a] // 2):
                ang = pos[a] * theta ** (-(2.0 * j) / dims[a])
                u, w = float(vec[2 * pair]), float(vec[2 * pair + 1])
                out[2 * pair] = u * math.cos(ang) - w * math.sin(ang)
                out[2 * pair + 1] = u * math.sin(ang) + w * math.cos(ang)
                pair += 1
        return out

    O = np.zeros((nq, H, D))
    Pm = np.zeros((nq, H, nk))
    for h in range(H):
        kr = [rot(k_raw[t, h], k_pos[t]) for t in range(nk)]
        for n in range(nq):
            qr = rot(q_raw[n, h], q_pos[n])
            sc = []
            for t in range(nk):
                ok = k_is_cache[t] or (not causal) or (k_blk[t] <= q_blk[n])
                if ok:
                    sc.append(sum(qr[d] * kr[t][d] for d in range(D)) / math.sqrt(D))
                else:
                    sc.append(None)
            m = max(s for s in sc if s is not None)
            e = [math.exp(s - m) if s is not None else 0.0 for s in sc]
            z = sum(e)
            for t in range(nk):
                Pm[n, h, t] = e[t] / z
                for d in range(D):
                    O[n, h, d] += e[t] / z * float(v[t, h, d])
    return O, Pm


def _tiny_case(seed, C, n_cache, Fb=1, Hh=2, Ww=3, H=2, dims=(4, 2, 2)):
    rng = np.random.default_rng(seed)
    D = sum(dims)
    L = Fb * Hh * Ww
    first_inflight = n_cache
    kv_g = list(range(n_cache + C))
    infl = list(range(first_inflight, first_inflight + C))
    q = [rng.standard_normal((L, H, D)) for _ in infl]
    k = [rng.standard_normal((L, H, D)) for _ in kv_g]
    v = [rng.standard_normal((L, H, D)) for _ in kv_g]
    states = [orc.CLEAN] * n_cache + [orc.NOISY] * C
    return dict(L=L, H=H, D=D, dims=dims, Fb=Fb, Hh=Hh, Ww=Ww, kv_g=kv_g, infl=infl,
                q=q, k=k, v=v, states=states)


def _run_oracle(c, mode, theta=10000.0, return_probs=False):
    pos = lambda g: orc.token_positions(g, c["Fb"], c["Hh"], c["Ww"])
    qr = [orc.rope3d(x, pos(g), c["dims"], theta) for x, g in zip(c["q"], c["infl"])]
    kr = [orc.rope3d(x, pos(g), c["dims"], theta) for x, g in zip(c["k"], c["kv_g"])]
    vis = orc.visibility(c["states"], c["kv_g"], c["infl"], mode)
    return orc.cascade_attention(qr, kr, c["v"], vis, return_probs=return_probs), vis


@pytest.mark.parametrize("mode", [orc.BIDIRECTIONAL, orc.BLOCK_CAUSAL])
@pytest.mark.parametrize("seed,C,n_cache", [(0, 3, 2), (1, 1, 1), (2, 2, 0)])
def test_brute_force_tiny(mode, seed, C, n_cache):
    c = _tiny_case(seed, C, n_cache)
    (outs, probs), vis = _run_oracle(c, mode, theta=50.0, return_probs=True)
    L = c["L"]
    pos = lambda g: [tuple(int(x) for x in p) for p in orc.token_positions(g, c["Fb"], c["Hh"], c["Ww"])]
    # positions recomputed by hand: frame = Fb*g + n // (Hh*Ww) etc.
    for g in c["kv_g"]:
        for n, p in enumerate(pos(g)):
            assert p == (c["Fb"] * g + n // (c["Hh"] * c["Ww"]), (n // c["Ww"]) % c["Hh"], n % c["Ww"])
    q_raw = np.concatenate(c["q"]); k_raw = np.concatenate(c["k"]); v = np.concatenate(c["v"])
    q_blk = [g for g in c["infl"] for _ in range(L)]
    k_blk = [g for g in c["kv_g"] for _ in range(L)]
    q_pos = [p for g in c["infl"] for p in pos(g)]
    k_pos = [p for g in c["kv_g"] for p in pos(g)]
    k_is_cache = [s == orc.CLEAN for s in c["states"] for _ in range(L)]
    O, Pm = brute_force(q_raw, k_raw, v, q_blk, k_blk, q_pos, k_pos, k_is_cache, c["dims"], 50.0,
                        causal=(mode == orc.BLOCK_CAUSAL))
    for i in range(C):
        np.testing.assert_allclose(outs[i], O[i * L:(i + 1) * L], rtol=0, atol=1e-12)
        # scatter the oracle's visible-key probabilities back to the full key axis
        full = np.zeros((L, c["H"], len(k_blk)))
        cols = np.concatenate([np.arange(r * L, (r + 1) * L) for r in range(len(c["kv_g"])) if vis[i, r]])
        full[:, :, cols] = probs[i]
        np.testing.assert_allclose(full, Pm[i * L:(i + 1) * L], rtol=0, atol=1e-13)


# --------------------------------------------------------------------------- attention pins

def _textbook(q, K, V):
    """softmax(QK^T/sqrt(D))V per head with a library softmax."""
    D = q.shape[-1]
    s = np.einsum("nhd,mhd->hnm", q, K) / math.sqrt(D)
    return np.einsum("hnm,mhd->nhd", softmax(s, axis=-1), V)


def test_all_visible_equals_full_attention():
    c = _tiny_case(3, 3, 2, Fb=2, Hh=3, Ww=4, H=3, dims=(8, 4, 4))
    outs, vis = _run_oracle(c, orc.BIDIRECTIONAL)
    assert vis.all()
    pos = lambda g: orc.token_positions(g, c["Fb"], c["Hh"], c["Ww"])
    K = np.concatenate([orc.rope3d(x, pos(g), c["dims"], 10000.0) for x, g in zip(c["k"], c["kv_g"])])
    V = np.concatenate(c["v"])
    for i, g in enumerate(c["infl"]):
        qi = orc.rope3d(c["q"][i], pos(g), c["dims"], 10000.0)
        np.testing.assert_allclose(outs[i], _textbook(qi, K, V), atol=1e-13)


def test_single_inflight_block_is_plain_block_causal():
    """Cascade P1 reduces to the block-causal pipeline (Fig. 7 caption): with one
    in-flight block both modes agree and equal full attention over [cache | self]."""
    c = _tiny_case(4, 1, 3, Fb=1, Hh=3, Ww=3)
    o_bi, _ = _run_oracle(c, orc.BIDIRECTIONAL)
    o_ca, _ = _run_oracle(c, orc.BLOCK_CAUSAL)
    np.testing.assert_array_equal(o_bi[0], o_ca[0])
    pos = lambda g: orc.token_positions(g, c["Fb"], c["Hh"], c["Ww"])
    K = np.concatenate([orc.rope3d(x, pos(g), c["dims"], 10000.0) for x, g in zip(c["k"], c["kv_g"])])
    q0 = orc.rope3d(c["q"][0], pos(c["infl"][0]), c["dims"], 10000.0)
    np.testing.assert_allclose(o_bi[0], _textbook(q0, K, np.concatenate(c["v"])), atol=1e-13)


@pytest.mark.parametrize("mode", [orc.BIDIRECTIONAL, orc.BLOCK_CAUSAL])
def test_probabilities_sum_to_one(mode):
    c = _tiny_case(5, 3, 2)
    (outs, probs), _ = _run_oracle(c, mode, return_probs=True)
    for p in probs:
        assert (p >= 0).all()
        np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-14)


@pytest.mark.parametrize("mode", [orc.BIDIRECTIONAL, orc.BLOCK_CAUSAL])
def test_constant_v_gives_constant_output(mode):
    c = _tiny_case(6, 3, 1)
    const = np.linspace(-1, 2, c["D"])
    c["v"] = [np.broadcast_to(const, x.shape).copy() for x in c["v"]]
    outs, _ = _run_oracle(c, mode)
    for o in outs:
        np.testing.assert_allclose(o, np.broadcast_to(const, o.shape), atol=1e-13)


@pytest.mark.parametrize("mode", [orc.BIDIRECTIONAL, orc.BLOCK_CAUSAL])
def test_zero_q_gives_mean_of_visible_v(mode):
    """Q = 0 makes softmax uniform, so O is the mean of the visible V rows: this
    checks the *number* of visible keys per mode, (cache + C) L vs (cache + i + 1) L."""
    n_cache, C = 2, 4
    c = _tiny_case(7, C, n_cache)
    c["q"] = [np.zeros_like(x) for x in c["q"]]
    outs, _ = _run_oracle(c, mode)
    for i, o in enumerate(outs):
        n_blocks = n_cache + (C if mode == orc.BIDIRECTIONAL else i + 1)
        mean = np.concatenate(c["v"][:n_blocks]).mean(axis=0)
        np.testing.assert_allclose(o, np.broadcast_to(mean, o.shape), atol=1e-13)


def test_kv_block_permutation_invariance():
    c = _tiny_case(8, 3, 3)
    outs, _ = _run_oracle(c, orc.BLOCK_CAUSAL)
    perm = [4, 0, 5, 2, 1, 3]
    d = dict(c)
    for key in ("k", "v", "kv_g", "states"):
        d[key] = [c[key][p] for p in perm]
    outs_p, _ = _run_oracle(d, orc.BLOCK_CAUSAL)
    for a, b in zip(outs, outs_p):
        np.testing.assert_allclose(a, b, atol=1e-13)


def test_block_causal_equals_bidirectional_on_truncated_pool():
    n_cache, C = 2, 4
    c = _tiny_case(9, C, n_cache)
    o_ca, _ = _run_oracle(c, orc.BLOCK_CAUSAL)
    for i in range(C):
        d = dict(c)
        keep = n_cache + i + 1
        for key in ("k", "v", "kv_g", "states"):
            d[key] = c[key][:keep]
        d["q"], d["infl"] = c["q"][:i + 1], c["infl"][:i + 1]
        o_bi, _ = _run_oracle(d, orc.BIDIRECTIONAL)
        np.testing.assert_allclose(o_ca[i], o_bi[i], atol=1e-13)


def test_row_subset_matches_full():
    c = _tiny_case(10, 2, 2, Fb=2, Hh=3, Ww=4)
    pos = lambda g: orc.token_positions(g, c["Fb"], c["Hh"], c["Ww"])
    qr = [orc.rope3d(x, pos(g), c["dims"], 1e4) for x, g in zip(c["q"], c["infl"])]
    kr = [orc.rope3d(x, pos(g), c["dims"], 1e4) for x, g in zip(c["k"], c["kv_g"])]
    vis = orc.visibility(c["states"], c["kv_g"], c["infl"], orc.BLOCK_CAUSAL)
    full = orc.cascade_attention(qr, kr, c["v"], vis)
    rows = [np.array([0, 5, 23]), np.array([7])]
    part = orc.cascade_attention(qr, kr, c["v"], vis, rows=rows, row_chunk=2)
    for f, p, r in zip(full, part, rows):
        np.testing.assert_allclose(p, f[r], atol=1e-14)


# --------------------------------------------------------------------------- RoPE pins

DIMS = (44, 42, 42)


def test_rope_preserves_norm():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((50, 3, 128))
    pos = rng.integers(0, 200, size=(50, 3))
    y = orc.rope3d(x, pos, DIMS, 10000.0)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    # pairwise too: each (even, odd) pair keeps its own norm
    np.testing.assert_allclose(y[..., 0::2] ** 2 + y[..., 1::2] ** 2,
                               x[..., 0::2] ** 2 + x[..., 1::2] ** 2, rtol=1e-12, atol=1e-14)


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((20, 2, 128)); k = rng.standard_normal((30, 2, 128))
    pq = rng.integers(0, 60, size=(20, 3)); pk = rng.integers(0, 60, size=(30, 3))
    shift = np.array([[17, 5, 29]])
    s0 = np.einsum("nhd,mhd->hnm", orc.rope3d(q, pq, DIMS, 1e4), orc.rope3d(k, pk, DIMS, 1e4))
    s1 = np.einsum("nhd,mhd->hnm", orc.rope3d(q, pq + shift, DIMS, 1e4),
                   orc.rope3d(k, pk + shift, DIMS, 1e4))
    np.testing.assert_allclose(s0, s1, atol=1e-10)
    # and it does depend on the difference: shifting only K changes scores
    s2 = np.einsum("nhd,mhd->hnm", orc.rope3d(q, pq, DIMS, 1e4), orc.rope3d(k, pk + shift, DIMS, 1e4))
    assert np.abs(s2 - s0).max() > 1e-2


def test_rope_identity_at_origin():
    x = np.random.default_rng(2).standard_normal((4, 2, 128))
    np.testing.assert_array_equal(orc.rope3d(x, np.zeros((4, 3), dtype=np.int64), DIMS, 1e4), x)


def test_rope_reduces_to_textbook_1d():
    """With all dims on one axis: x_pair * exp(i * pos * theta^(-2j/D)) (complex form)."""
    rng = np.random.default_rng(3)
    D = 16
    x = rng.standard_normal((9, 1, D))
    pos = np.zeros((9, 3), dtype=np.int64); pos[:, 0] = np.arange(9) * 3
    y = orc.rope3d(x, pos, (D, 0, 0), 100.0)
    z = (x[..., 0::2] + 1j * x[..., 1::2]) * np.exp(
        1j * pos[:, 0][:, None, None] * 100.0 ** (-np.arange(D // 2) * 2.0 / D)[None, None, :])
    np.testing.assert_allclose(y[..., 0::2], z.real, atol=1e-13)
    np.testing.assert_allclose(y[..., 1::2], z.imag, atol=1e-13)


def test_rope_one_hot_closed_form_and_axis_layout():
    """(1,0) in pair j of axis a maps to (cos phi, sin phi), phi = pos_a * theta^(-2 j_a / D_a);
    checks which head-dim range belongs to which axis and that the other axes' positions do not leak."""
    theta = 10000.0
    pos = np.array([[7, 11, 13]])
    first = 0
    for a, Da in enumerate(DIMS):
        for ja in (0, 1, Da // 2 - 1):
            x = np.zeros((1, 1, 128)); x[0, 0, first + 2 * ja] = 1.0
            y = orc.rope3d(x, pos, DIMS, theta)
            phi = pos[0, a] * theta ** (-2.0 * ja / Da)
            exp = np.zeros(128); exp[first + 2 * ja] = math.cos(phi); exp[first + 2 * ja + 1] = math.sin(phi)
            np.testing.assert_allclose(y[0, 0], exp, atol=1e-15)
            x = np.zeros((1, 1, 128)); x[0, 0, first + 2 * ja + 1] = 1.0
            y = orc.rope3d(x, pos, DIMS, theta)
            exp = np.zeros(128); exp[first + 2 * ja] = -math.sin(phi); exp[first + 2 * ja + 1] = math.cos(phi)
            np.testing.assert_allclose(y[0, 0], exp, atol=1e-15)
        first += Da


def test_token_positions_layout():
    p = orc.token_positions(2, 3, 30, 52)
    assert p.shape == (4680, 3)
    assert tuple(p[0]) == (6, 0, 0) and tuple(p[51]) == (6, 0, 51) and tuple(p[52]) == (6, 1, 0)
    assert tuple(p[1560]) == (7, 0, 0) and tuple(p[-1]) == (8, 29, 51)
    assert len({tuple(r) for r in p}) == 4680


# --------------------------------------------------------------------------- visibility pins

def test_visibility_structure_and_counts():
    n_cache, C = 6, 5
    states = [orc.SINK] + [orc.CLEAN] * (n_cache - 1) + [orc.NOISY] * C
    kv_g = list(range(n_cache + C))
    infl = kv_g[n_cache:]
    bi = orc.visibility(states, kv_g, infl, orc.BIDIRECTIONAL)
    ca = orc.visibility(states, kv_g, infl, orc.BLOCK_CAUSAL)
    assert bi.shape == (C, n_cache + C) and bi.all()
    assert ca[:, :n_cache].all()
    np.testing.assert_array_equal(ca[:, n_cache:], np.tril(np.ones((C, C), dtype=np.uint8)))
    L = 4680
    assert int(bi.sum()) * L * L == 1_204_632_000
    assert int(ca.sum()) * L * L == 985_608_000
    # a resident noisy block that is not part of this forward is invisible
    v = orc.visibility(states, kv_g, infl[1:], orc.BIDIRECTIONAL)
    assert not v[:, n_cache].any() and v[:, n_cache + 1:].all()


# --------------------------------------------------------------------------- cache state machine pins

def _rollout(S, W, C, steps, switch_at=None):
    T = (1000, 750, 500, 250, 0)
    cache = orc.KVCacheOracle(S, W, C, pages_per_block=37, heads=12)
    epoch = 0
    log = []
    for step in range(steps):
        if switch_at is not None and step == switch_at:
            epoch += 1
            before = cache.snapshot()
            cache.retag(epoch)
            after = cache.snapshot()
            # the prompt switch touches only the epoch of NOISY entries (Sec. 3.5)
            for x, y in zip(before, after):
                assert x[:4] == y[:4]
                assert y[4] == (epoch if x[2] == orc.NOISY else x[4])
        b, batch, slots = orc.rollout_step(cache, step, T, epoch)
        snap_mid = cache.snapshot()
        evicted = orc.rollout_finish(cache, b, batch)
        log.append(dict(step=step, b=b, batch=batch, slots=slots, evicted=evicted,
                        mid=snap_mid, end=cache.snapshot()))
    return cache, log


@pytest.mark.parametrize("S,W", [(1, 6), (0, 6), (0, 2), (1, 1)])
def test_cache_invariants_over_rollout(S, W):
    C = 5
    cache, log = _rollout(S, W, C, steps=60, switch_at=20)
    ring = W + C
    prev_evicted_slot = None
    for e in log:
        for snap in (e["mid"], e["end"]):
            slots = [s[0] for s in snap]
            assert len(set(slots)) == len(slots)                          # injective
            blocks = [s[1] for s in snap]
            assert len(set(blocks)) == len(blocks)
            for s in snap:
                if s[1] < S:
                    assert s[0] == s[1]                                   # sink block pinned to its slot
                    assert s[2] in (orc.NOISY, orc.SINK)
                else:
                    assert s[0] >= S and s[2] != orc.SINK
            live = sorted(s[1] for s in snap if s[1] >= S)
            assert not live or live == list(range(live[0], live[0] + len(live)))  # contiguous g range
            assert len(live) <= ring
        assert sum(1 for s in e["end"] if s[2] == orc.CLEAN) <= W
        # in-flight tags: oldest block is cleanest (Alg. 1: block b+i runs at T[tau-i])
        ts = [t for _, t in e["batch"]]
        assert ts == sorted(ts)
        step = e["step"]
        assert len(e["batch"]) == min(step, 4) + 1
        if step >= 4:
            assert ts == [0, 250, 500, 750, 1000]
        # the block admitted this step lands in the slot freed by the previous eviction
        if prev_evicted_slot is not None:
            assert e["slots"][-1] == prev_evicted_slot
        prev_evicted_slot = None
        if e["evicted"] is not None:
            g = e["evicted"]
            prev_evicted_slot = S + ((g - S) % ring)
            assert g == e["b"] - W                                        # the oldest of the window
    # slot pattern of the in-flight blocks repeats with the ring period
    for e in log[10:40]:
        later = log[e["step"] + ring]
        assert e["slots"] == later["slots"]
    # eviction starts exactly when S + W blocks are cached
    first_evict = next(e["step"] for e in log if e["evicted"] is not None)
    assert first_evict == 4 + S + W


def test_cache_errors_leave_state_unchanged():
    c = orc.KVCacheOracle(1, 2, 2, 3, 2)
    c.append(0, 1000, 0); c.append(1, 1000, 0)
    snap = c.snapshot()
    with pytest.raises(orc.CacheError):
        c.append(1 + 4, 1000, 0)          # slot of block 5 == slot of block 1, still held
    with pytest.raises(orc.CacheError):
        c.evict(7)
    with pytest.raises(orc.CacheError):
        c.promote(3)
    assert c.snapshot() == snap
    c.promote(0)
    with pytest.raises(orc.CacheError):
        c.evict(0)                        # sink refuses
    with pytest.raises(orc.CacheError):
        c.promote(0)
    with pytest.raises(orc.CacheError):
        c.append(0, 0, 0)
    c.promote(1); c.evict(1)
    assert [s[1] for s in c.snapshot()] == [0]


def test_page_index_is_a_bijection():
    c = orc.KVCacheOracle(1, 6, 5, 37, 12)
    idx = {c.page_index(s, p, h) for s in range(c.n_slots) for p in range(37) for h in range(12)}
    assert idx == set(range(c.n_slots * 37 * 12))
    assert c.page_index(0, 0, 1) == 1 and c.page_index(0, 1, 0) == 12 and c.page_index(1, 0, 0) == 37 * 12


def test_kv_order():
    cache, _ = _rollout(1, 6, 5, steps=15)
    b, batch, _ = orc.rollout_step(cache, 15, (1000, 750, 500, 250, 0), 0)
    order, states, slots = cache.kv_order([g for g, _ in batch])
    assert order == [0] + list(range(b - 6, b)) + list(range(b, b + 5))
    assert states == [orc.SINK] + [orc.CLEAN] * 6 + [orc.NOISY] * 5
    assert slots == [cache.slot_of(g) for g in order]


def test_algorithm1_trace_counts_golden():
    """Alg. 1 with G = 5 and B blocks runs B+4 iterations with batch sizes
    1,2,3,4,5,...,5,4,3,2,1 and forwards every block exactly 5 times, in the order
    t3,t2,t1,t0,tc; block b+i is always one step noisier than b+i-1."""
    with open(os.path.join(HERE, "golden", "alg1_batch_sizes_B13_G5.txt")) as f:
        golden = [int(x) for line in f if not line.startswith("#") for x in line.split()]
    tr = orc.algorithm1_trace(13, 5)
    assert [len(t[3]) for t in tr] == golden
    assert len(tr) == 13 + 4 and sum(golden) == 5 * 13
    seen = {}
    for b, tau, d, batch in tr:
        assert batch[0][0] == b
        for i, (g, ti) in enumerate(batch):
            seen.setdefault(g, []).append(ti)
            assert ti == batch[0][1] - i
    assert seen == {g: [0, 1, 2, 3, 4] for g in range(13)}
    for B in (5, 7, 20):   # the listing never bounds the ramp-up by B, so it needs B >= G
        tr = orc.algorithm1_trace(B, 5)
        assert len(tr) == B + 4
        assert sum(len(t[3]) for t in tr) == 5 * B


def test_schedule_matches_algorithm1_trace():
    T = (1000, 750, 500, 250, 0)
    tr = orc.algorithm1_trace(30, 5)
    for step in range(20):
        b, batch = orc.cascade_schedule(step, T, 5)
        assert b == tr[step][0]
        assert batch == [(g, T[ti]) for g, ti in tr[step][3]]


def test_layer_linear_against_the_definition_and_special_cases():
    """x @ w.T: brute force over every (m, n, k) on a tiny case, identity and one-hot weights
    (which pick columns of x), and linearity in each argument."""
    rng = np.random.default_rng(3)
    x, w = rng.standard_normal((5, 7)), rng.standard_normal((4, 7))
    brute = np.zeros((5, 4))
    for m in range(5):
        for n in range(4):
            for k in range(7):
                brute[m, n] += x[m, k] * w[n, k]
    np.testing.assert_allclose(orc.layer_linear(x, w), brute, rtol=1e-13, atol=1e-13)
    np.testing.assert_array_equal(orc.layer_linear(x, np.eye(7)), x)
    onehot = np.zeros((2, 7)); onehot[0, 3] = 1.0; onehot[1, 6] = -2.0
    np.testing.assert_array_equal(orc.layer_linear(x, onehot), np.stack([x[:, 3], -2.0 * x[:, 6]], axis=1))
    x2, w2 = rng.standard_normal((5, 7)), rng.standard_normal((4, 7))
    np.testing.assert_allclose(orc.layer_linear(x + 2 * x2, w), orc.layer_linear(x, w) + 2 * orc.layer_linear(x2, w), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(orc.layer_linear(x, w - w2), orc.layer_linear(x, w) - orc.layer_linear(x, w2), rtol=1e-12, atol=1e-12)
    assert orc.layer_linear(x, w).shape == (5, 4)            # [rows, out], weights stored [out, in]


def test_cascade_type_schedule_properties():
    """lag 1 is Alg. 1's batch sequence; for any lag every block visits every timestep once, in
    order, one per iteration; consecutive blocks are `lag` iterations apart; at most
    ceil(|T| / lag) blocks are in flight: 1, 2, 3, 5 for lag 5, 3, 2, 1 (P1..P4)."""
    T = 5
    for B in (5, 8, 13):
        assert orc.cascade_type_schedule(B, T, 1) == [batch for _, _, _, batch in orc.algorithm1_trace(B, 5)]
    for lag, width in ((5, 1), (3, 2), (2, 3), (1, 5), (4, 2)):
        sch = orc.cascade_type_schedule(7, T, lag)
        assert max(len(b) for b in sch) == width == -(-T // lag)
        seen = {}
        for n, batch in enumerate(sch):
            assert batch == sorted(batch)                               # oldest block first
            for j, idx in batch:
                seen.setdefault(j, []).append((n, idx))
        assert sorted(seen) == list(range(7))
        for j, visits in seen.items():
            assert [idx for _, idx in visits] == list(range(T))
            assert [n for n, _ in visits] == list(range(lag * j, lag * j + T))
        assert len(sch) == lag * 6 + T
    assert orc.cascade_type_schedule(3, T, 5) == [[(j, i)] for j in range(3) for i in range(T)]   # sequential
