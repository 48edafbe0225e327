"""Shared test plumbing: run one cascade forward on the GPU path and on the oracle.

The two sides meet only here, on the same seeded inputs from `workloads`; neither
imports the other.
"""
from __future__ import annotations

import numpy as np

import workloads as W
from oracle import cascade_oracle as orc

BF16_MAX_ABS = 2e-2     # tolerances of the bf16 path against the fp64 oracle
BF16_REL_L2 = 5e-3
F32_MAX_ABS = 2e-5      # fp32 path, relative to max(1, max|ref|): fp32 rounding over <= ~10^3 keys
F32_REL_L2 = 1e-5


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    a = a.astype(np.float64).ravel(); b = b.astype(np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def assert_close(gpu: np.ndarray, ref: np.ndarray, dtype: str, what: str = "",
                 max_abs_lim: float | None = None, rel_lim: float | None = None,
                 bound: np.ndarray | None = None, **kw) -> None:
    """The two spec bars (max-abs and relative L2 over the compared tensor) and, when
    `bound` is given, |gpu - ref| <= bound element by element (see attention_element_bound)."""
    max_abs_lim = kw.get("max_abs", max_abs_lim)
    rel_lim = kw.get("rel", rel_lim)
    err = np.abs(gpu.astype(np.float64) - ref)
    max_abs = float(err.max())
    r = rel_l2(gpu, ref)
    if dtype == "bf16":
        lim_abs, lim_rel = BF16_MAX_ABS, BF16_REL_L2
    else:
        lim_abs, lim_rel = F32_MAX_ABS * max(1.0, float(np.abs(ref).max())), F32_REL_L2
    lim_abs = lim_abs if max_abs_lim is None else max_abs_lim
    lim_rel = lim_rel if rel_lim is None else rel_lim
    worst = ""
    if bound is not None:
        ratio = err / bound
        worst = f" max err/bound={float(ratio.max()):.3f}"
    print(f"[parity] {what}: max_abs={max_abs:.3e} (<= {lim_abs:.1e}) rel_l2={r:.3e} (<= {lim_rel:.1e}){worst}", flush=True)
    assert max_abs <= lim_abs and r <= lim_rel, f"{what}: max_abs={max_abs:.3e} rel_l2={r:.3e}"
    if bound is not None:
        bad = np.argwhere(err > bound)
        assert len(bad) == 0, (f"{what}: {len(bad)} of {err.size} elements outside the per-element bound, first at "
                               f"{tuple(int(x) for x in bad[0])}: gpu={gpu[tuple(bad[0])]!r} ref={ref[tuple(bad[0])]!r} "
                               f"bound={bound[tuple(bad[0])]!r}")


# --------------------------------------------------------------------------- per-element error model
# What separates the bf16 kernel's result from the fp64 definition, term by term (first order).
# A rounding to bf16 (8 significant bits) is off by at most half a unit in the last place: 2^-8
# relative at the bottom of a binade, 2^-9 at the top; taken as uniform within that, its relative
# variance averaged over a binade is E2 = (2^-8)^2 / 3 / 2.
#   * the result is rounded to bf16 once: <= 2^-8 |o|;
#   * every probability is rounded to bf16 before the PV product, while the normalising row sum is
#     taken over the unrounded probabilities (the usual flash-attention arithmetic): the rounding
#     errors e_k, independent from key to key, move output element d by sum_k p_k e_k v_kd;
#   * the logits are formed from bf16 operands: the rotated K is stored as bf16, the rotated Q is
#     stored as bf16 and rounded once more after the multiplication by log2(e)/sqrt(D).  Each rounding
#     perturbs logit s_k = sum_d q_d k_kd / sqrt(D) by sum_d q_d k_kd e_d / sqrt(D): variance
#     E2 * sum_d q_d^2 k_kd^2 / D per rounding, three roundings; a perturbation ds_k of a logit moves
#     output element d by p_k ds_k (v_kd - o_d) (the softmax derivative);
#   * so  var(o_d) = sum_k p_k^2 (var(ds_k) (v_kd - o_d)^2 + E2 v_kd^2) .
# The bound allows 8 standard deviations of that sum (a tensor has ~10^6 elements, the terms are
# bounded, and the perturbations that come from rounding Q are shared by the keys of a row rather
# than independent, which the margin has to absorb) plus the final rounding.  fp32 accumulation
# (2^-24 per addition) is far below either term.
E2_BF16 = (2.0 ** -8) ** 2 / 6.0
N_SIGMA = 8.0


def attention_element_bound(o, p, q_rot, k_rot, v, logit_roundings: int = 3):
    """o [n, D] fp64 oracle output of one head, p [n, keys] its probabilities, q_rot [n, D] and
    k_rot [keys, D] the rotated queries / keys (fp64), v [keys, D].  Returns the bound [n, D]."""
    D = q_rot.shape[1]
    p2 = p * p
    ps = p2 * ((logit_roundings * E2_BF16 / D) * ((q_rot * q_rot) @ (k_rot * k_rot).T))    # p_k^2 var(ds_k)
    v2 = v * v
    var_o = ps @ v2 - 2.0 * o * (ps @ v) + o * o * ps.sum(axis=1, keepdims=True) + E2_BF16 * (p2 @ v2)
    return 1.01 * 2.0 ** -8 * np.abs(o) + N_SIGMA * np.sqrt(np.maximum(var_o, 0.0)) + 1e-30


# --------------------------------------------------------------------------- oracle side

def oracle_forward(w: W.Workload, q, k, v, cached_g, inflight_g, mode, rows=None, heads=None):
    """q [C*L,H,D], k/v [(n_cached+C)*L,H,D] in storage dtype, KV blocks ordered cached then in-flight.
    Returns list of O_i (fp64) for the in-flight blocks; `heads` restricts to a head subset."""
    L = w.block_tokens
    hs = slice(None) if heads is None else list(heads)
    kv_g = list(cached_g) + list(inflight_g)
    pos = lambda g: orc.token_positions(g, w.frames_per_block, w.grid_h, w.grid_w)
    qb = [orc.rope3d(W.to_f64(x[:, hs]), pos(g), w.rope_dims, w.rope_theta)
          for x, g in zip(W.split_blocks(q, L), inflight_g)]
    if rows is not None:
        qb = [x[np.asarray(r)] for x, r in zip(qb, rows)]
    kb = [orc.rope3d(W.to_f64(x[:, hs]), pos(g), w.rope_dims, w.rope_theta)
          for x, g in zip(W.split_blocks(k, L), kv_g)]
    vb = [W.to_f64(x[:, hs]) for x in W.split_blocks(v, L)]
    states = [orc.CLEAN] * len(cached_g) + [orc.NOISY] * len(inflight_g)
    vis = orc.visibility(states, kv_g, inflight_g, mode)
    return orc.cascade_attention(qb, kb, vb, vis)


def oracle_forward_bounded(w: W.Workload, q, k, v, cached_g, inflight_g, mode, rows=None, heads=None,
                            head_chunk: int = 1, row_chunk: int = 1024, kv=None):
    """oracle_forward plus the per-element bound of attention_element_bound, head_chunk heads (one
    at a time keeps every per-head slice the oracle takes contiguous) and at most row_chunk query
    rows per block at a time so that the probabilities (rows x keys per head) stay small.  Returns (list of O_i, list of bound_i), each [rows_i, len(heads), D].
    kv = (kv_g, states, k_blocks, v_blocks) overrides the "cached then in-flight" layout
    (rollouts: blocks in the order and state of the cache); q may be a list of per-block tensors."""
    L = w.block_tokens
    heads = list(range(w.heads)) if heads is None else list(heads)
    pos = lambda g: orc.token_positions(g, w.frames_per_block, w.grid_h, w.grid_w)
    if kv is None:
        kv_g = list(cached_g) + list(inflight_g)
        states = [orc.CLEAN] * len(cached_g) + [orc.NOISY] * len(inflight_g)
        k_blocks, v_blocks = W.split_blocks(k, L), W.split_blocks(v, L)
    else:
        kv_g, states, k_blocks, v_blocks = kv
    q_blocks = q if isinstance(q, (list, tuple)) else W.split_blocks(q, L)
    n_q = len(inflight_g)
    vis = orc.visibility(states, kv_g, inflight_g, mode)
    rows = [np.arange(L) for _ in range(n_q)] if rows is None else [np.asarray(r, dtype=np.int64) for r in rows]
    outs = [np.empty((len(r), len(heads), w.head_dim)) for r in rows]
    bounds = [np.empty((len(r), len(heads), w.head_dim)) for r in rows]
    for c0 in range(0, len(heads), head_chunk):
        hs = heads[c0:c0 + head_chunk]
        q_rot = [orc.rope3d(W.to_f64(x[:, hs]), pos(g), w.rope_dims, w.rope_theta) for x, g in zip(q_blocks, inflight_g)]
        kb = [orc.rope3d(W.to_f64(x[:, hs]), pos(g), w.rope_dims, w.rope_theta) for x, g in zip(k_blocks, kv_g)]
        vb = [W.to_f64(x[:, hs]) for x in v_blocks]
        for i in range(n_q):
            sel = [r for r in range(len(kv_g)) if vis[i, r]]
            kcat = [np.concatenate([kb[r][:, j] for r in sel]) for j in range(len(hs))]
            vcat = [np.concatenate([vb[r][:, j] for r in sel]) for j in range(len(hs))]
            for r0 in range(0, len(rows[i]), row_chunk):
                rr = rows[i][r0:r0 + row_chunk]
                # the oracle on query block i alone: its row of the visibility matrix, its rows rr
                o, p = orc.cascade_attention([q_rot[i]], kb, vb, vis[i:i + 1], rows=[rr], return_probs=True)
                for j in range(len(hs)):
                    outs[i][r0:r0 + len(rr), c0 + j] = o[0][:, j]
                    bounds[i][r0:r0 + len(rr), c0 + j] = attention_element_bound(
                        o[0][:, j], p[0][:, j], q_rot[i][rr][:, j], kcat[j], vcat[j])
    return outs, bounds


# --------------------------------------------------------------------------- GPU side

def to_torch(x: np.ndarray, dtype: str, device="cuda:0"):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(x.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(x).to(device)


def from_torch(t, dtype: str) -> np.ndarray:
    import torch
    if dtype == "bf16":
        return W.bf16_bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16))
    return t.cpu().numpy()


def gpu_setup(w: W.Workload, k, v, cached_g, inflight_g, timesteps=None):
    """Create a pool, publish cached blocks (append + promote) and in-flight blocks."""
    from paper_2511_20426_amd.runner import CascadePool
    pool = CascadePool.for_workload(w)
    L = w.block_tokens
    kt, vt = to_torch(k, w.dtype), to_torch(v, w.dtype)
    kv_g = list(cached_g) + list(inflight_g)
    ts = timesteps or [0] * len(inflight_g)
    for j, g in enumerate(kv_g):
        cached = j < len(cached_g)
        pool.append(g, 0 if cached else ts[j - len(cached_g)], 0, kt[j * L:(j + 1) * L], vt[j * L:(j + 1) * L])
        if cached:
            pool.ctx.kv_cache_promote(g)
    return pool


def gpu_forward(w: W.Workload, pool, q, inflight_g, mode):
    """Rotate Q (blocks must be consecutive in the video) and run the cascade forward."""
    import torch
    assert list(inflight_g) == list(range(inflight_g[0], inflight_g[0] + len(inflight_g)))
    qt = to_torch(q, w.dtype)
    qr = pool.rope(qt, w.frames_per_block * inflight_g[0])
    # the result buffer starts as NaN: a row the launch failed to write cannot pass for a result
    out = pool.forward(qr, inflight_g, mode, out=torch.full_like(qr, float("nan")))
    torch.cuda.synchronize()
    return from_torch(out, w.dtype)


def gpu_forward_rope(w: W.Workload, pool, q, inflight_g, mode, packed: bool = True):
    """The forward on unrotated queries (cascade_attn_forward_rope); with packed=True q is handed
    over as the strided q part of a [tokens, 3, H, D] tensor, as a QKV projection leaves it."""
    import torch
    qt = to_torch(q, w.dtype)
    if packed:
        box = torch.full((qt.shape[0], 3, qt.shape[1], qt.shape[2]), float("nan"), dtype=qt.dtype, device=qt.device)
        box[:, 0] = qt
        qt = box[:, 0]
    out = pool.forward_rope(qt, inflight_g, mode, out=torch.full(tuple(qt.shape), float("nan"), dtype=qt.dtype,
                                                                  device=qt.device))
    torch.cuda.synchronize()
    return from_torch(out, w.dtype)


def gpu_forward_share(w: W.Workload, pool, q, inflight_g, mode, first, count):
    """The same for the queries of in-flight blocks first .. first+count-1 only
    (cascade_attn_forward_share); q is the whole [C*L, H, D] tensor, the result [count*L, H, D]."""
    import torch
    L = w.block_tokens
    qt = to_torch(np.ascontiguousarray(q[first * L:(first + count) * L]), w.dtype)
    qr = pool.rope(qt, w.frames_per_block * inflight_g[first])
    out = pool.forward(qr, inflight_g, mode, out=torch.full_like(qr, float("nan")), share=(first, count))
    torch.cuda.synchronize()
    return from_torch(out, w.dtype)


# --------------------------------------------------------------------------- pool decoding
# Written from the page format documented in include/cascade_attn.h.

_PERM = [0, 1, 2, 3, 8, 9, 10, 11, 4, 5, 6, 7, 12, 13, 14, 15]


def decode_bf16_pages(pool_bytes: np.ndarray, pair_index: int):
    """(K [128 tokens,128 dims], V [128 tokens,128 dims]) as bf16 bit patterns."""
    base = pair_index * 65536
    raw = pool_bytes[base:base + 65536].view(np.uint16).reshape(2, 128, 16, 8)   # page,row,pos,elem
    K = np.empty((128, 128), np.uint16)
    V = np.empty((128, 128), np.uint16)
    for r in range(128):
        for c in range(16):
            K[r, 8 * c:8 * c + 8] = raw[0, r, c ^ (r & 15)]
            chunk = raw[1, r, c ^ (r & 15)]                      # row r = dim, eight tokens
            for e in range(8):
                V[16 * (c // 2) + _PERM[8 * (c % 2) + e], r] = chunk[e]
    return K, V


def decode_f32_pages(pool_bytes: np.ndarray, pair_index: int, page_tokens: int, head_dim: int):
    n = page_tokens * head_dim
    raw = pool_bytes[pair_index * 2 * n * 4:(pair_index + 1) * 2 * n * 4].view(np.float32)
    return raw[:n].reshape(page_tokens, head_dim), raw[n:].reshape(page_tokens, head_dim)
