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
                 max_abs_lim: float | None = None, rel_lim: float | None = None, **kw) -> None:
    max_abs_lim = kw.get("max_abs", max_abs_lim)
    rel_lim = kw.get("rel", rel_lim)
    max_abs = float(np.abs(gpu.astype(np.float64) - ref).max())
    r = rel_l2(gpu, ref)
    if dtype == "bf16":
        lim_abs, lim_rel = BF16_MAX_ABS, BF16_REL_L2
    else:
        lim_abs, lim_rel = F32_MAX_ABS * max(1.0, float(np.abs(ref).max())), F32_REL_L2
    lim_abs = lim_abs if max_abs_lim is None else max_abs_lim
    lim_rel = lim_rel if rel_lim is None else rel_lim
    print(f"[parity] {what}: max_abs={max_abs:.3e} (<= {lim_abs:.1e}) rel_l2={r:.3e} (<= {lim_rel:.1e})", flush=True)
    assert max_abs <= lim_abs and r <= lim_rel, f"{what}: max_abs={max_abs:.3e} rel_l2={r:.3e}"


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
