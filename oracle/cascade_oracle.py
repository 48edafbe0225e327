"""CPU oracle for block-cascaded self-attention.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the hot path computes, written from
the paper's problem statement.  It shares no code with the HIP library and is
imported only by tests, the smoke check and the benchmark's cpu_baseline leg.
Every function is pinned by CPU tests against brute force, closed forms and
invariants; nothing here is "parity unpinned".

What is computed (paper passages):

* blocks of `Fb` latent frames; a block is bidirectional inside (Sec. 3.1, the
  paragraph on block-causal generation);
* several in-flight blocks at different denoising steps are batched into one
  forward and share attention (Sec. 3.2 last paragraph); their K/V live in one
  shared KV pool next to the clean cache of finished blocks (Sec. 3.3);
* across the cascade attention is bidirectional (Sec. 3.4) or block-causal
  (the causal P4 variant, Sec. 4.2; Sec. 3.2: block i attends to blocks i-k and itself);
* a rolling window of clean blocks with eviction of the oldest, optionally a
  sink block kept for ever (Sec. 2.3, Sec. 3.3);
* the per-iteration schedule of Algorithm 1 (block b+i runs at T[tau-i]);
* a prompt switch keeps every cached K/V as is (Sec. 3.5).

The paper never mentions rotary embeddings; they belong to the Wan-family DiT
it adapts.  Convention used here: head_dim is split into three runs of
consecutive (even, odd) pairs for the frame, row and column axes, pair j of an
axis with D_a dims has frequency theta**(-2j/D_a), positions are absolute
integer (frame, row, col) indices counted from 0.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BIDIRECTIONAL = 0
BLOCK_CAUSAL = 1

FREE, NOISY, CLEAN, SINK = 0, 1, 2, 3


# --------------------------------------------------------------------------- geometry

def token_positions(g: int, frames_per_block: int, grid_h: int, grid_w: int) -> np.ndarray:
    """(frame, row, col) of every token of block `g` (Sec. 3.2: block i holds
    consecutive latent frames).  Token order is frame-major, then row, then column."""
    L = frames_per_block * grid_h * grid_w
    n = np.arange(L, dtype=np.int64)
    f = frames_per_block * g + n // (grid_h * grid_w)
    y = (n % (grid_h * grid_w)) // grid_w
    x = n % grid_w
    return np.stack([f, y, x], axis=1)


# --------------------------------------------------------------------------- RoPE

def rope3d(x: np.ndarray, pos: np.ndarray, dims: Sequence[int], theta: float) -> np.ndarray:
    """Rotate x[n, H, D] by the 3-axis rotary embedding at integer positions pos[n, 3]."""
    x = np.asarray(x, dtype=np.float64)
    n, H, D = x.shape
    assert sum(dims) == D and all(d % 2 == 0 for d in dims)
    angle = np.zeros((n, D // 2), dtype=np.float64)
    first = 0
    for a, Da in enumerate(dims):
        j = np.arange(Da // 2, dtype=np.float64)
        freq = np.power(float(theta), -2.0 * j / Da) if Da else j
        angle[:, first:first + Da // 2] = pos[:, a:a + 1].astype(np.float64) * freq[None, :]
        first += Da // 2
    c = np.cos(angle)[:, None, :]
    s = np.sin(angle)[:, None, :]
    u, v = x[..., 0::2], x[..., 1::2]
    y = np.empty_like(x)
    y[..., 0::2] = u * c - v * s
    y[..., 1::2] = u * s + v * c
    return y


# --------------------------------------------------------------------------- visibility

def visibility(kv_state: Sequence[int], kv_g: Sequence[int], inflight_g: Sequence[int],
               mode: int) -> np.ndarray:
    """vis[i, r]: may query block inflight_g[i] attend to KV block r?

    Clean cached blocks and the sink are visible to every in-flight block
    (Sec. 3.3).  An in-flight KV block is visible to every in-flight query block
    in bidirectional mode (Sec. 3.4); in block-causal mode only if it is not
    later in the video than the query block (Sec. 3.2).  A resident NOISY block
    that is not part of this forward is not visible.
    """
    infl = list(inflight_g)
    vis = np.zeros((len(infl), len(kv_g)), dtype=np.uint8)
    for i, gi in enumerate(infl):
        for r, (st, gr) in enumerate(zip(kv_state, kv_g)):
            if st in (CLEAN, SINK):
                vis[i, r] = 1
            elif st == NOISY and gr in infl:
                vis[i, r] = 1 if (mode == BIDIRECTIONAL or gr <= gi) else 0
    return vis


# --------------------------------------------------------------------------- attention

def cascade_attention(q_blocks: Sequence[np.ndarray], k_blocks: Sequence[np.ndarray],
                      v_blocks: Sequence[np.ndarray], vis: np.ndarray,
                      scale: Optional[float] = None, rows: Optional[Sequence[np.ndarray]] = None,
                      return_probs: bool = False, row_chunk: int = 512):
    """Masked softmax attention, by its definition, in fp64.

    q_blocks[i]  [Lq_i, H, D]  rotated queries of in-flight block i
    k_blocks[r]  [L_r, H, D]   rotated keys of KV block r;  v_blocks[r] likewise (not rotated)
    vis[i, r]    block-pair visibility; inside a visible pair every token pair is visible
    rows[i]      optional row indices: compute only those query rows of block i
    Returns a list of O_i [rows_i, H, D]; with return_probs also the list of
    P_i [rows_i, H, n_visible_keys_i].
    """
    outs, probs = [], []
    for i, q in enumerate(q_blocks):
        q = np.asarray(q, dtype=np.float64)
        if rows is not None:
            q = q[np.asarray(rows[i], dtype=np.int64)]
        sel = [r for r in range(len(k_blocks)) if vis[i, r]]
        K = np.concatenate([np.asarray(k_blocks[r], dtype=np.float64) for r in sel], axis=0)
        V = np.concatenate([np.asarray(v_blocks[r], dtype=np.float64) for r in sel], axis=0)
        n, H, D = q.shape
        sc = 1.0 / math.sqrt(D) if scale is None else scale
        o = np.empty((n, H, D), dtype=np.float64)
        p_all = np.empty((n, H, K.shape[0]), dtype=np.float64) if return_probs else None
        for h in range(H):
            Kh = np.ascontiguousarray(K[:, h, :])
            Vh = np.ascontiguousarray(V[:, h, :])
            for r0 in range(0, n, row_chunk):
                s = (q[r0:r0 + row_chunk, h, :] @ Kh.T) * sc
                s -= s.max(axis=1, keepdims=True)
                p = np.exp(s)
                p /= p.sum(axis=1, keepdims=True)
                o[r0:r0 + row_chunk, h, :] = p @ Vh
                if return_probs:
                    p_all[r0:r0 + row_chunk, h, :] = p
        outs.append(o)
        probs.append(p_all)
    return (outs, probs) if return_probs else outs


# --------------------------------------------------------------------------- cache state machine

class CacheError(Exception):
    pass


class KVCacheOracle:
    """Integer model of the shared KV pool: sink slots, rolling window, in-flight blocks.

    Slots 0..S+W+C-1.  Block g < S is a sink block and lives in slot g for ever;
    any other block lives in slot S + ((g - S) mod (W + C)).  Live non-sink
    blocks always form a contiguous range of at most W + C block indices (W clean
    ones behind C in flight), so the ring never collides (Sec. 3.3: fixed window,
    oldest block leaves; sink block kept in an external cache).
    """

    def __init__(self, sink_blocks: int, window_blocks: int, max_inflight: int,
                 pages_per_block: int, heads: int):
        self.S, self.W, self.C = sink_blocks, window_blocks, max_inflight
        self.P, self.H = pages_per_block, heads
        self.n_slots = self.S + self.W + self.C
        self.block = [-1] * self.n_slots
        self.state = [FREE] * self.n_slots
        self.timestep = [0] * self.n_slots
        self.epoch = [0] * self.n_slots

    def slot_of(self, g: int) -> int:
        if g < 0:
            raise CacheError("negative block id")
        if g < self.S:
            return g
        return self.S + ((g - self.S) % (self.W + self.C))

    def page_index(self, slot: int, page: int, head: int) -> int:
        """Physical page of (slot, page-in-block, head) in the pool."""
        return (slot * self.P + page) * self.H + head

    def find(self, g: int) -> int:
        s = self.slot_of(g)
        if self.state[s] == FREE or self.block[s] != g:
            raise CacheError(f"block {g} not resident")
        return s

    def append(self, g: int, timestep: int, epoch: int) -> int:
        s = self.slot_of(g)
        if self.state[s] != FREE and self.block[s] != g:
            raise CacheError(f"slot {s} still holds block {self.block[s]}")
        if self.state[s] in (CLEAN, SINK):
            raise CacheError("block already finished")
        self.block[s], self.state[s], self.timestep[s], self.epoch[s] = g, NOISY, timestep, epoch
        return s

    def promote(self, g: int) -> None:
        s = self.find(g)
        if self.state[s] != NOISY:
            raise CacheError("only a NOISY block can be promoted")
        self.state[s] = SINK if g < self.S else CLEAN

    def evict(self, g: int) -> None:
        s = self.find(g)
        if self.state[s] == SINK:
            raise CacheError("the sink is never evicted")
        self.block[s], self.state[s], self.timestep[s], self.epoch[s] = -1, FREE, 0, 0

    def retag(self, new_epoch: int) -> None:
        """Prompt switch (Sec. 3.5): only the prompt tag of partially denoised
        blocks changes; clean K/V and the slot map stay."""
        for s in range(self.n_slots):
            if self.state[s] == NOISY:
                self.epoch[s] = new_epoch

    def snapshot(self) -> List[Tuple[int, int, int, int, int]]:
        """(slot, block, state, timestep, epoch) of every occupied slot, by slot."""
        return [(s, self.block[s], self.state[s], self.timestep[s], self.epoch[s])
                for s in range(self.n_slots) if self.state[s] != FREE]

    def clean_window(self) -> List[int]:
        return sorted(self.block[s] for s in range(self.n_slots) if self.state[s] == CLEAN)

    def kv_order(self, inflight_g: Sequence[int]):
        """KV sequence of one forward: sink blocks, clean window by ascending block
        index, then the in-flight blocks by ascending index.  Returns (g, state, slot) lists."""
        sink = sorted(self.block[s] for s in range(self.n_slots) if self.state[s] == SINK)
        order = sink + self.clean_window() + sorted(inflight_g)
        slots = [self.find(g) for g in order]
        return order, [self.state[s] for s in slots], slots


def cascade_schedule(step: int, timesteps: Sequence[int], width: int, n_blocks: Optional[int] = None):
    """Blocks in flight at 0-based iteration `step` of Alg. 1 with `width` = G =
    len(timesteps) parallel blocks: [(block index, timestep)] oldest first, and the
    primary block b.  Block b+i runs at T[tau-i]: older blocks are cleaner."""
    nT = len(timesteps)
    assert width == nT, "Alg. 1 is self-consistent only for G = |T|"
    tau = min(step, nT - 1)
    b = max(0, step - (nT - 1))
    batch = []
    for i in range(0, min(tau, width - 1) + 1):
        if n_blocks is not None and b + i >= n_blocks:
            break
        batch.append((b + i, timesteps[tau - i]))
    return b, batch


def rollout_step(cache: KVCacheOracle, step: int, timesteps: Sequence[int], epoch: int):
    """One cascade iteration on the cache metadata, in Alg. 1's order: publish the
    in-flight blocks' K/V (append), [attention happens here], then the block that
    just ran at tc becomes clean, the window drops its oldest block if it now
    exceeds W.  This function does the part before attention and returns
    (primary block b, batch, slots); `rollout_finish` does the part after it."""
    b, batch = cascade_schedule(step, timesteps, cache.C)
    slots = [cache.append(g, t, epoch) for g, t in batch]
    return b, batch, slots


def rollout_finish(cache: KVCacheOracle, b: int, batch) -> Optional[int]:
    """After attention: promote the primary block if it ran at tc, evict the oldest
    window block if more than W are clean.  Returns the evicted block or None."""
    evicted = None
    if batch[0][1] == 0:                      # primary block completed the cache step tc
        cache.promote(b)
        win = cache.clean_window()
        if len(win) > cache.W:
            evicted = win[0]
            cache.evict(evicted)
    return evicted


def algorithm1_trace(n_blocks: int, n_gpus: int, n_timesteps: int = 5):
    """State trace of Alg. 1: list of (b, tau, d, batch) per iteration, batch =
    [(block, timestep index)]."""
    b = tau = d = 0
    trace = []
    while d >= 0:
        batch = [(b + i, tau - i) for i in range(min(d, n_gpus - 1) + 1)]
        trace.append((b, tau, d, batch))
        if tau - 0 == n_timesteps - 1:        # block b just ran the cache step tc
            b += 1
            if b + d >= n_blocks:
                d -= 1
        else:
            d = min(d + 1, n_gpus - 1)
            tau += 1
    return trace


def layer_linear(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """The linear maps either side of the attention inside a layer (QKV projection, output
    projection): y[m, n] = sum_k x[m, k] w[n, k], weights stored [out, in].  fp64; the paper
    treats these as part of the generator G_theta (Sec. 3.1) and gives no more than that."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    assert x.ndim == 2 and w.ndim == 2 and x.shape[1] == w.shape[1]
    return x @ w.T


def cascade_type_schedule(n_blocks: int, n_timesteps: int, lag: int):
    """Batches of a cascade in which block j enters `lag` iterations after block j-1 and moves
    one timestep per iteration: iteration n forwards every block j with 0 <= n - lag*j <
    n_timesteps at timestep index n - lag*j.  lag = 1 is Alg. 1 (five blocks in flight for the
    five-entry timestep list); lag = n_timesteps is sequential block-causal generation (P1 of the
    ablation, Sec. 4.2 / Fig. 7); lag 3 and 2 give the 2- and 3-block cascades.  Written as the
    closed form, not as a state machine.  Returns [[(block, timestep index), ...] per iteration]."""
    out = []
    for n in range(lag * (n_blocks - 1) + n_timesteps):
        out.append([(j, n - lag * j) for j in range(n_blocks) if 0 <= n - lag * j < n_timesteps])
    return out
