"""The per-element error bound of the attention comparisons (tests/_harness.py), checked on the CPU.

Two things have to hold for the bound to mean anything: a computation that makes exactly the
roundings the bound is derived from (bf16 rotated Q and K, Q rounded again after the scale, bf16
probabilities under a row sum of the unrounded ones, against an exponent reference that is
not the row maximum, one bf16 rounding of the result; everything else exact) must stay inside it, with
room; and a single wrong output element, far too small to move the two norm bars, must fall
outside it.  No GPU is involved: the "kernel" here is a numpy model of the roundings.
"""
import math

import numpy as np
import pytest

import workloads as W
from oracle import cascade_oracle as orc
from tests import _harness as Hn


def _bf16(x):
    return W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))).astype(np.float64)


def _rounding_model(w, q, k, v, cached, infl, mode):
    """Masked attention with the roundings of a bf16 kernel and nothing else."""
    L, D = w.block_tokens, w.head_dim
    pos = lambda g: orc.token_positions(g, w.frames_per_block, w.grid_h, w.grid_w)
    kv_g = list(cached) + list(infl)
    c = math.log2(math.e) / math.sqrt(D)
    qb = [_bf16(_bf16(orc.rope3d(W.to_f64(x), pos(g), w.rope_dims, w.rope_theta)) * np.float32(c))
          for x, g in zip(W.split_blocks(q, L), infl)]
    kb = [_bf16(orc.rope3d(W.to_f64(x), pos(g), w.rope_dims, w.rope_theta)) for x, g in zip(W.split_blocks(k, L), kv_g)]
    vb = [W.to_f64(x) for x in W.split_blocks(v, L)]
    vis = orc.visibility([orc.CLEAN] * len(cached) + [orc.NOISY] * len(infl), kv_g, infl, mode)
    outs = []
    for i in range(len(infl)):
        sel = [r for r in range(len(kv_g)) if vis[i, r]]
        K = np.concatenate([kb[r] for r in sel]); V = np.concatenate([vb[r] for r in sel])
        o = np.empty_like(qb[i])
        for h in range(w.heads):
            s = qb[i][:, h] @ K[:, h].T                       # log2 units
            # the reference of a row is the maximum of its first 32 keys, as in a kernel that does
            # not track the running maximum: the dominant probabilities are not powers of two
            p = np.exp2(s - s[:, :32].max(axis=1, keepdims=True))
            o[:, h] = (_bf16(p) @ V[:, h]) / p.sum(axis=1, keepdims=True)
        outs.append(_bf16(o))
    return outs


@pytest.mark.parametrize("mode", [orc.BIDIRECTIONAL, orc.BLOCK_CAUSAL])
@pytest.mark.parametrize("scale", [0.5, 2.0])
def test_bound_admits_the_rounding_model_and_rejects_one_wrong_element(mode, scale):
    w = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=2, grid_h=7, grid_w=9, n_cached=2, n_inflight=2)
    q, k, v = W.draw_config(w, seed=3, scale=scale)
    cached, infl = [0, 1], [2, 3]
    ref, bound = Hn.oracle_forward_bounded(w, q, k, v, cached, infl, mode, row_chunk=64)
    ref, bound = np.concatenate(ref), np.concatenate(bound)
    got = np.concatenate(_rounding_model(w, q, k, v, cached, infl, mode))
    ratio = np.abs(got - ref) / bound
    print(f"rounding model: max err/bound {ratio.max():.3f}, rms {np.sqrt((ratio ** 2).mean()):.3f}, "
          f"rel L2 {Hn.rel_l2(got, ref):.2e}")
    assert ratio.max() <= 0.8                     # 8 sigma allowed; the model stays well inside
    assert np.sqrt((ratio ** 2).mean()) >= 0.05   # and the bound is not slack by orders of magnitude
    grow = (scale / 0.5) ** 1.3
    Hn.assert_close(got, ref, "bf16", "rounding model", bound=bound, max_abs=2e-2 * grow, rel=5e-3 * grow)
    # one element wrong by 6 %: a single bad key or a slip in one lane; the norms do not notice
    bad = got.copy()
    typical = np.abs(np.abs(ref) - 2.0 * np.median(np.abs(ref)))
    idx = tuple(int(x) for x in np.unravel_index(np.argmin(typical), ref.shape))
    bad[idx] *= 1.06
    Hn.assert_close(bad, ref, "bf16", "one wrong element, norm bars only", max_abs=2e-2 * grow, rel=5e-3 * grow)
    with pytest.raises(AssertionError, match="per-element bound"):
        Hn.assert_close(bad, ref, "bf16", "one wrong element", bound=bound, max_abs=2e-2 * grow, rel=5e-3 * grow)


def test_bound_follows_the_number_of_keys():
    """The rounding terms average out over the keys a row sees: with near-uniform weights the
    statistical part of the bound falls like 1 / sqrt(keys)."""
    w1 = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=1, grid_h=4, grid_w=8, n_cached=0, n_inflight=1)
    w4 = W.small_variant(W.CONFIGS["c3_wan1p3b_cascade5"], heads=1, grid_h=4, grid_w=8, n_cached=3, n_inflight=1)
    stat = []
    for w, cached, infl in ((w1, [], [0]), (w4, [0, 1, 2], [3])):
        q, k, v = W.draw_config(w, seed=5)
        ref, bound = Hn.oracle_forward_bounded(w, q, k, v, cached, infl, orc.BIDIRECTIONAL)
        stat.append(float(np.mean(bound[0] - 1.01 * 2.0 ** -8 * np.abs(ref[0]))))
    assert 1.6 < stat[0] / stat[1] < 2.5          # 4x the keys: about half
