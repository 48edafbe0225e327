"""Seeded synthetic workloads for block-cascaded attention.

This module is the only code shared by the CPU oracle's tests and the GPU
path's tests/benchmarks.  It holds *no* arithmetic of the method (no RoPE, no
softmax, no cache-slot rule): only shapes, seeded Gaussian draws and dtype
plumbing (fp32 <-> bf16 bit patterns, round-to-nearest-even).

Shapes follow the Wan-family video DiT the paper adapts (Sec. 3.1): blocks of 3
latent frames, a 5-entry timestep list {t3,t2,t1,t0,tc} (Sec. 3.2, Alg. 1).
The real activations (trained checkpoints, benchmark prompts) are not
available; N(0,1)*input_scale tensors of the same shape stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Tuple

import numpy as np

# Timestep list of Alg. 1 (T = {t3, t2, t1, t0, tc}); numeric values are the
# usual 4-step distillation schedule plus the cache step tc = 0 (Sec. 3.2).
TIMESTEPS: Tuple[int, ...] = (1000, 750, 500, 250, 0)


@dataclass(frozen=True)
class Workload:
    name: str
    heads: int
    head_dim: int
    frames_per_block: int
    grid_h: int
    grid_w: int
    rope_dims: Tuple[int, int, int]   # (frame, row, col) split of head_dim
    rope_theta: float
    sink_blocks: int                  # S
    window_blocks: int                # W  (clean cached blocks kept)
    max_inflight: int                 # C  (cascade width)
    n_cached: int                     # cached blocks present in the one-shot configs
    n_inflight: int                   # in-flight blocks in the one-shot configs
    dtype: str                        # "f32" | "bf16"
    input_scale: float
    seed: int
    page_tokens: int

    @property
    def block_tokens(self) -> int:    # L
        return self.frames_per_block * self.grid_h * self.grid_w

    @property
    def pages_per_block(self) -> int:  # P
        return -(-self.block_tokens // self.page_tokens)

    @property
    def n_q(self) -> int:
        return self.n_inflight * self.block_tokens

    @property
    def n_kv(self) -> int:
        return (self.n_cached + self.n_inflight) * self.block_tokens

    def visible_pairs(self, block_causal: bool = False) -> int:
        """(query, key) pairs per head that the mask leaves visible."""
        L = self.block_tokens
        if not block_causal:
            return self.n_q * self.n_kv
        return sum(L * (self.n_cached + i + 1) * L for i in range(self.n_inflight))

    def flops(self, block_causal: bool = False) -> float:
        """Algorithmic flops of one forward: QK^T and PV, 2 flops per multiply-add."""
        return 4.0 * self.head_dim * self.visible_pairs(block_causal) * self.heads


_WAN = dict(head_dim=128, frames_per_block=3, grid_h=30, grid_w=52,
            rope_dims=(44, 42, 42), rope_theta=10000.0, dtype="bf16",
            input_scale=0.5, seed=0, page_tokens=128, window_blocks=6,
            max_inflight=5, sink_blocks=0)

CONFIGS = {
    # tiny fp32 case: the oracle finishes in well under a second
    "c1_tiny_f32": Workload(name="c1_tiny_f32", heads=2, head_dim=64, frames_per_block=3,
                            grid_h=6, grid_w=8, rope_dims=(24, 20, 20), rope_theta=10000.0,
                            sink_blocks=0, window_blocks=2, max_inflight=1, n_cached=2,
                            n_inflight=1, dtype="f32", input_scale=1.0, seed=0, page_tokens=48),
    # Wan-1.3B shape, sequential baseline: one in-flight block (cascade P1, Fig. 7)
    "c2_wan1p3b_seq": Workload(name="c2_wan1p3b_seq", heads=12, n_cached=6, n_inflight=1, **_WAN),
    # Wan-1.3B shape, 5-block cascade
    "c3_wan1p3b_cascade5": Workload(name="c3_wan1p3b_cascade5", heads=12, n_cached=6,
                                    n_inflight=5, **_WAN),
    # Wan-14B shape, 5-block cascade: the headline configuration
    "c4_wan14b_cascade5": Workload(name="c4_wan14b_cascade5", heads=40, n_cached=6,
                                   n_inflight=5, **_WAN),
    # long rollout at the 1.3B shape: 1 sink block + 6-block sliding window
    "c5_wan1p3b_rollout": Workload(name="c5_wan1p3b_rollout", heads=12, n_cached=0, n_inflight=5,
                                   **{**_WAN, "sink_blocks": 1}),
}


def small_variant(w: Workload, *, heads: int, grid_h: int, grid_w: int, **kw) -> Workload:
    """Same structure as `w` on a smaller token grid (parity cases the oracle finishes quickly)."""
    return replace(w, name=w.name + "_small", heads=heads, grid_h=grid_h, grid_w=grid_w, **kw)


# --------------------------------------------------------------------------- dtype plumbing

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even; inputs are finite."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(x: np.ndarray) -> np.ndarray:
    """Exact widening of a stored tensor (fp32 values or bf16 bit patterns) to float64."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


def store(x_f32: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 draws to the storage type both sides consume (fp32 array or bf16 bits)."""
    if dtype == "bf16":
        return f32_to_bf16_bits(x_f32)
    if dtype == "f32":
        return np.ascontiguousarray(x_f32, dtype=np.float32)
    raise ValueError(dtype)


# --------------------------------------------------------------------------- draws

def draw_qkv(w: Workload, n_q_blocks: int, n_kv_blocks: int, seed: int | None = None,
             scale: float | None = None, k_ramp: tuple | None = None):
    """Q [n_q_blocks*L,H,D], K and V [n_kv_blocks*L,H,D] in storage dtype.

    Draw order Q, K, V from numpy's default_rng(seed), float32 standard normal
    times `scale`.  KV blocks are ordered oldest first: cached blocks, then the
    in-flight ones; K is pre-RoPE.  k_ramp=(a, b): K token n is multiplied by a geometric ramp
    from a (oldest token) to b (newest), so that the largest logit of a row keeps growing (or
    shrinking) along the KV sequence; k_ramp=(a, b, "step") switches from a to b half way.
    """
    rng = np.random.default_rng(w.seed if seed is None else seed)
    s = np.float32(w.input_scale if scale is None else scale)
    L, H, D = w.block_tokens, w.heads, w.head_dim
    out = []
    for which, nb in enumerate((n_q_blocks, n_kv_blocks, n_kv_blocks)):
        x = rng.standard_normal((nb * L, H, D), dtype=np.float32)
        x *= s
        if which == 1 and k_ramp is not None:
            if len(k_ramp) > 2 and k_ramp[2] == "step":      # a for the older half, b for the newer
                ramp = np.where(np.arange(nb * L) < (nb * L) // 2, k_ramp[0], k_ramp[1]).astype(np.float32)
            else:
                ramp = np.geomspace(k_ramp[0], k_ramp[1], nb * L).astype(np.float32)
            x *= ramp[:, None, None]
        out.append(store(x, w.dtype))
    return tuple(out)


def draw_config(w: Workload, seed: int | None = None, scale: float | None = None,
                k_ramp: tuple | None = None):
    """The one-shot configurations: Q for the in-flight blocks, K/V for cached + in-flight."""
    return draw_qkv(w, w.n_inflight, w.n_cached + w.n_inflight, seed, scale, k_ramp)


def draw_step_block(w: Workload, step: int, i: int, seed: int | None = None):
    """Long-rollout recipe: (Q, K, V) [L,H,D] of the i-th in-flight block of cascade step `step`,
    each from its own generator seeded by (seed + step, i, tensor) so that any block of any step
    can be drawn without the others."""
    base = (w.seed if seed is None else seed) + step
    out = []
    for which in range(3):
        rng = np.random.default_rng([base, i, which])
        x = rng.standard_normal((w.block_tokens, w.heads, w.head_dim), dtype=np.float32)
        x *= np.float32(w.input_scale)
        out.append(store(x, w.dtype))
    return tuple(out)


def split_blocks(x: np.ndarray, L: int) -> List[np.ndarray]:
    assert x.shape[0] % L == 0
    return [x[i * L:(i + 1) * L] for i in range(x.shape[0] // L)]


def sample_rows(L: int, n_random: int, seed: int, tile_edges=(128, 256), offsets=(0,)) -> np.ndarray:
    """Deterministic row sample inside one block: first/last two rows, rows either
    side of every multiple of the given tile sizes, plus seeded random rows.  `offsets`: where
    tiles start relative to the block's first row (0: tiles counted from the block's own first
    row; o: from a row o before it, as when tiles run across several blocks laid end to end)."""
    rows = {0, 1, L - 2, L - 1}
    for t in tile_edges:
        for off in offsets:
            for e in range(t - off % t, L, t):
                rows.update((e - 1, e))
    rng = np.random.default_rng(seed)
    rows.update(int(r) for r in rng.integers(0, L, size=n_random))
    return np.array(sorted(r for r in rows if 0 <= r < L), dtype=np.int64)


def draw_linear(m_rows: int, n_out: int, k_in: int, seed: int, x_scale: float = 1.0):
    """Activations X [m_rows, k_in] ~ N(0,1) * x_scale and weights W [n_out, k_in] ~ N(0,1) / sqrt(k_in)
    (outputs of unit scale, as after a normalised layer input), both rounded to bf16 bit patterns."""
    rng = np.random.default_rng([seed, m_rows, n_out, k_in])
    x = rng.standard_normal((m_rows, k_in), dtype=np.float32) * np.float32(x_scale)
    w = rng.standard_normal((n_out, k_in), dtype=np.float32) * np.float32(1.0 / np.sqrt(k_in))
    return store(x, "bf16"), store(w, "bf16")
