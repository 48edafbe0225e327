"""Algorithm 1 as a driver over the library: the scheduler's batches are published to the cache,
attended, and retired, for a rollout of B blocks.

The denoiser around the attention (projections, MLPs, the re-noising operator Psi, the decoder)
is not part of this library; the caller supplies it as `qkv_fn`, which returns the pre-RoPE
Q/K/V of one block at one timestep, and receives the attention output through `out_fn`.  This
module only sequences library calls; it holds no arithmetic.

Run as a program it measures the steady-state iteration rate of the attention hot path in the
paper's streaming protocol (Sec. 4, implementation details: the mean over the 8th and 9th block
of a 13-block rollout), with synthetic Q/K/V:

    python -m paper_2511_20426_amd.rollout --workload c4_wan14b_cascade5
"""
from __future__ import annotations

import argparse
import json
from dataclasses import dataclass, field, replace
from typing import Callable, List, Optional, Sequence, Tuple

import torch

from . import binding as B
from .runner import CascadePool


@dataclass
class IterationRecord:
    iteration: int
    batch: List[Tuple[int, int, int]]          # (block, timestep index, timestep), oldest first
    emitted: int                               # block whose t0 prediction is the output, or -1
    completed: int                             # block that ran tc and became clean, or -1
    evicted: int                               # block dropped from the window, or -1
    ms: Optional[float] = None                 # device time of the iteration (events), if timed
    events: Optional[tuple] = field(default=None, repr=False, compare=False)   # (start, end) until run() reads them


@dataclass
class CascadeRollout:
    """Drives `pool` through Alg. 1 for `n_blocks` blocks.

    qkv_fn(block, timestep_index, iteration, position) -> (q, k, v), each [L, H, D] on the device.
    out_fn(block, timestep_index, o) receives that block's slice of the attention output.
    """
    pool: CascadePool
    n_blocks: int
    timesteps: Sequence[int]
    qkv_fn: Optional[Callable] = None
    out_fn: Optional[Callable] = None
    # optional stand-ins for the layer around the attention, run inside the timed region:
    # batch_qkv_fn(batch) -> [(q, k, v) per block] (e.g. one QKV projection for the whole batch),
    # post_fn(o) (e.g. the output projection)
    batch_qkv_fn: Optional[Callable] = None
    post_fn: Optional[Callable] = None
    # publish_fn(batch, epoch) -> packed unrotated queries [n * L, H, D]: publishes the batch's K/V
    # itself (layer_qkv_publish: one launch for projection and cache write); the queries then go to
    # the attention kernel as they are (cascade_attn_forward_rope).  Replaces qkv_fn / batch_qkv_fn.
    publish_fn: Optional[Callable] = None
    mode: int = B.CA_BIDIRECTIONAL
    window_blocks: Optional[int] = None        # clean blocks kept; default: the pool's window
    epoch: int = 0
    lag: Optional[int] = None                  # None: Alg. 1; otherwise the lagged cascade (5, 3, 2: P1..P3)
    timed: bool = False
    records: List[IterationRecord] = field(default_factory=list)

    def __post_init__(self):
        self.sched = B.Scheduler(self.n_blocks, len(self.timesteps), list(self.timesteps), lag=self.lag)
        cfg = self.pool.cfg
        self._window = cfg.window_blocks if self.window_blocks is None else self.window_blocks
        if self._window > cfg.window_blocks:
            raise ValueError("window_blocks exceeds the pool's window")
        self._sink = cfg.sink_blocks
        self._clean: List[int] = []            # clean non-sink blocks, oldest first
        L, H, D = self.pool.block_tokens, self.pool.heads, self.pool.head_dim
        from .runner import torch_dtype
        dt = torch_dtype(self.pool.dtype)
        n = len(self.timesteps)
        self._qr = torch.empty((n * L, H, D), dtype=dt, device=self.pool.device)
        self._o = torch.empty_like(self._qr)

    def step(self) -> Optional[IterationRecord]:
        """One iteration of Alg. 1; None once the rollout is over."""
        batch = self.sched.batch()
        if not batch:
            return None
        pool, L = self.pool, self.pool.block_tokens
        it = self.sched.state()[3]
        if self.timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if self.batch_qkv_fn is None and self.publish_fn is None:
            staged = [self.qkv_fn(g, ti, it, i) for i, (g, ti, _) in enumerate(batch)]
        if self.timed:
            e0.record()
        n = len(batch)
        infl = [g for g, _, _ in batch]
        if self.publish_fn is not None:
            q = self.publish_fn(batch, self.epoch)
            o = pool.forward_rope(q[:n * L], infl, self.mode, out=self._o[:n * L])
        else:
            if self.batch_qkv_fn is not None:
                staged = self.batch_qkv_fn(batch)
            ks, vs = [s[1] for s in staged], [s[2] for s in staged]
            if all(t.stride() == ks[0].stride() for t in ks + vs):
                pool.append_batch(infl, [t for _, _, t in batch], self.epoch, ks, vs)
            else:                                  # one launch needs one set of strides
                for (g, ti, t), k, v in zip(batch, ks, vs):
                    pool.append(g, t, self.epoch, k, v)
            for i, ((g, ti, t), (q, k, v)) in enumerate(zip(batch, staged)):
                # each block's queries are rotated from wherever they live into the packed tensor
                pool.rope(q, pool.frames_per_block * g, out=self._qr[i * L:(i + 1) * L])
            o = pool.forward(self._qr[:n * L], infl, self.mode, out=self._o[:n * L])
        if self.post_fn is not None:
            self.post_fn(o)
        emitted, completed = self.sched.advance()
        evicted = -1
        if completed >= 0:
            pool.ctx.kv_cache_promote(completed)
            if completed >= self._sink:
                self._clean.append(completed)
                if len(self._clean) > self._window:
                    evicted = self._clean.pop(0)
                    pool.ctx.kv_cache_evict(evicted)
        if self.timed:
            e1.record()
        if self.out_fn is not None:
            for i, (g, ti, _) in enumerate(batch):
                self.out_fn(g, ti, o[i * L:(i + 1) * L])
        rec = IterationRecord(it, batch, emitted, completed, evicted)
        if self.timed:
            rec.events = (e0, e1)
        self.records.append(rec)
        return rec

    def run(self) -> List[IterationRecord]:
        while self.step() is not None:
            pass
        if self.timed:
            torch.cuda.synchronize(self.pool.device)
            for r in self.records:
                if r.events is not None:
                    r.ms = r.events[0].elapsed_time(r.events[1])
                    r.events = None
        return self.records


def streaming_rate(records: Sequence[IterationRecord], blocks=(7, 8)) -> float:
    """Iterations per second over the iterations that emit the given blocks (0-based ids 7 and 8
    are the 8th and 9th block: the steady state of a 13-block rollout, Sec. 4)."""
    ms = [r.ms for r in records if r.emitted in blocks]
    if len(ms) != len(blocks) or any(m is None for m in ms):
        raise ValueError("rollout too short or not timed")
    return 1e3 * len(ms) / sum(ms)


def main(argv=None) -> None:
    import workloads as W
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--workload", default="c4_wan14b_cascade5")
    ap.add_argument("--blocks", type=int, default=13)
    ap.add_argument("--window", type=int, default=None,
                    help="clean blocks kept (default: the workload's; 2 gives the 7-block window "
                         "of the paper's accounting, 5 in flight + 2 cached)")
    ap.add_argument("--mode", choices=("bidirectional", "block_causal"), default="bidirectional")
    ap.add_argument("--repeats", type=int, default=3)
    ap.add_argument("--lag", type=int, default=None,
                    help="iterations between consecutive blocks: 5, 3, 2, 1 = the 1-, 2-, 3-, 5-block cascades "
                         "P1..P4 (default: Alg. 1 = 1)")
    ap.add_argument("--layer", action="store_true",
                    help="include the QKV and output projections (synthetic weights) in every iteration")
    ap.add_argument("--three-launches", action="store_true",
                    help="with --layer: the projection publishes K/V itself and the attention kernel rotates Q "
                         "(layer_qkv_publish, cascade_attn_forward_rope) instead of five launches per iteration")
    a = ap.parse_args(argv)
    w = W.CONFIGS[a.workload]
    dev = torch.device("cuda:0")
    pool_w = w if a.window is None else replace(w, window_blocks=a.window, n_cached=a.window)
    L, H, D = w.block_tokens, w.heads, w.head_dim
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    # one set of synthetic Q/K/V per cascade position, reused every iteration (values do not
    # change the work; the rollout's data movement and launches are the real ones)
    bank = [tuple((torch.randn((L, H, D), generator=gen, device=dev) * w.input_scale).to(torch.bfloat16)
                  for _ in range(3)) for _ in range(len(W.TIMESTEPS))]
    mode = B.CA_BIDIRECTIONAL if a.mode == "bidirectional" else B.CA_BLOCK_CAUSAL
    hooks = {}
    if a.layer:
        from .runner import linear
        width = H * D
        x = (torch.randn((len(W.TIMESTEPS) * L, width), generator=gen, device=dev)).to(torch.bfloat16)
        w_qkv = (torch.randn((3 * width, width), generator=gen, device=dev) / width ** 0.5).to(torch.bfloat16)
        w_out = (torch.randn((width, width), generator=gen, device=dev) / width ** 0.5).to(torch.bfloat16)
        qkv = torch.empty((len(W.TIMESTEPS) * L, 3, H, D), dtype=torch.bfloat16, device=dev)
        y = torch.empty((len(W.TIMESTEPS) * L, width), dtype=torch.bfloat16, device=dev)

        def batch_qkv_fn(batch):
            n = len(batch) * L
            linear(x[:n], w_qkv, out=qkv[:n].view(n, 3 * width))
            return [(qkv[i * L:(i + 1) * L, 0], qkv[i * L:(i + 1) * L, 1], qkv[i * L:(i + 1) * L, 2])
                    for i in range(len(batch))]

        def post_fn(o):
            n = o.shape[0]
            linear(o.view(n, width), w_out, out=y[:n])

        q_packed = torch.empty((len(W.TIMESTEPS) * L, H, D), dtype=torch.bfloat16, device=dev)
        current = {}

        def publish_fn(batch, epoch):
            n = len(batch) * L
            return current["pool"].qkv_publish(x[:n], w_qkv, [g for g, _, _ in batch], [t for _, _, t in batch], epoch,
                                               q_out=q_packed[:n])

        if a.three_launches:
            hooks = dict(publish_fn=publish_fn, post_fn=post_fn)
        else:
            hooks = dict(batch_qkv_fn=batch_qkv_fn, post_fn=post_fn)
    rates, steady_ms = [], []
    for rep in range(a.repeats + 1):                      # first pass warms up
        pool = CascadePool.for_workload(pool_w)
        if a.layer:
            current["pool"] = pool
        ro = CascadeRollout(pool, a.blocks, W.TIMESTEPS, lambda g, ti, it, i: bank[i], mode=mode, timed=True, lag=a.lag, **hooks)
        recs = ro.run()
        if rep:
            rates.append(streaming_rate(recs))
            steady_ms.append([r.ms for r in recs if r.emitted in (7, 8)])
        del ro, pool
    window = pool_w.window_blocks
    print(json.dumps({
        "metric": "steady_state_cascade_iterations_per_s", "value": sum(rates) / len(rates),
        "unit": "iterations/s (one attention layer%s; one block of 3 latent frames emitted per iteration)"
                % ((" with its QKV and output projections" + (", three launches" if a.three_launches else "")) if a.layer else ""),
        "protocol": "mean over the iterations emitting the 8th and 9th block of a %d-block rollout" % a.blocks,
        "workload": w.name, "mode": a.mode, "clean_window_blocks": window, "lag": a.lag or 1,
        "blocks_per_s": a.blocks / (sum(r.ms for r in recs) * 1e-3),
        "iteration_ms": steady_ms, "iterations": len(recs), "data": "synthetic",
    }))


if __name__ == "__main__":
    main()
