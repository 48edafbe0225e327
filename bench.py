#!/usr/bin/env python3
"""Benchmark of the block-cascaded attention hot path on one MI355X.

A step is one cascade iteration of one self-attention layer at the Wan-14B shape in steady
state (6 clean cached blocks + 5 blocks in flight): publish the 5 in-flight blocks' K/V
(fused K-RoPE + page write), rotate Q and run the cascaded attention (one launch: the attention
kernel rotates the queries as it loads them; --two-launch-q takes the separate rope3d_apply),
then promote the block that completed the cache step, evict the oldest window block and move on
by one block.
Inputs are seeded synthetic N(0,1)*0.5 bf16 tensors already resident in HBM.

Prints ONE JSON line: whole-path TFLOP/s (algorithmic attention flops / step time), the
roofline of the dominant kernel (attention, MFMA-bound) from its own HIP-event timing, and
the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6        # MI355X dense bf16 MFMA: 256 CU x 4096 flop/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
# HBM bytes per attention launch at the Wan-14B shape, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# scaled by a 1 GiB copy (profiles/c4_wan14b_cascade5_hbm_traffic.txt): 4295.3 MB read + 259.6 MB written
# by the attention kernel, 26.2 + 8.3 MB by the merge of its split work items
ATTN_TRAFFIC_BYTES_C4 = 4.5894e9


def cpu_baseline(w, seconds_target=15.0):
    """The fp64 oracle, as it stands, on a bounded sample: a few heads, a slice of query rows
    of the first in-flight block against all visible keys (K rotation included)."""
    import numpy as np
    from oracle import cascade_oracle as orc
    import workloads as W
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    L, D = w.block_tokens, w.head_dim
    n_kv_blocks = w.n_cached + w.n_inflight
    heads, rows = 2, 2048
    rng = np.random.default_rng(0)
    total_flops, total_t = 0.0, 0.0
    pos = lambda g: orc.token_positions(g, w.frames_per_block, w.grid_h, w.grid_w)
    kv_g = list(range(n_kv_blocks))
    g_q = w.n_cached
    states = [orc.CLEAN] * w.n_cached + [orc.NOISY] * w.n_inflight
    vis = orc.visibility(states, kv_g, [g_q], orc.BIDIRECTIONAL)
    for _ in range(64):                        # until seconds_target of oracle time
        q = W.store(rng.standard_normal((L, heads, D), dtype=np.float32) * 0.5, "bf16")
        k = W.store(rng.standard_normal((n_kv_blocks * L, heads, D), dtype=np.float32) * 0.5, "bf16")
        v = W.store(rng.standard_normal((n_kv_blocks * L, heads, D), dtype=np.float32) * 0.5, "bf16")
        t0 = time.perf_counter()
        qb = [orc.rope3d(W.to_f64(q), pos(g_q), w.rope_dims, w.rope_theta)[:rows]]
        kb = [orc.rope3d(W.to_f64(x), pos(g), w.rope_dims, w.rope_theta)
              for x, g in zip(W.split_blocks(k, L), kv_g)]
        vb = [W.to_f64(x) for x in W.split_blocks(v, L)]
        orc.cascade_attention(qb, kb, vb, vis)
        total_t += time.perf_counter() - t0
        total_flops += 4.0 * D * rows * n_kv_blocks * L * heads
        if total_t >= seconds_target:
            break
    return {
        "value": total_flops / total_t / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
        "sample": f"fp64 numpy oracle, {total_flops / 1e9:.0f} GFLOP of the same shape in {total_t:.1f} s "
                  f"(query-row slices of one in-flight block x a few heads vs all {n_kv_blocks * L} keys, "
                  f"K/Q rotation included)",
    }


def time_attention_only(torch, W, B, w, modes, shares=(), launches=5, prepared=None):
    """Attention launches of workload `w` on a steady-state pool (n_cached clean blocks, the
    in-flight ones appended, Q rotated), timed with events around `launches` forwards after two
    warm-up calls.  Returns {label: {"ms", "TFLOP/s", "frac"}}; `shares`: also one device's share
    (queries of in-flight block i only) per mode.  prepared = (pool, in-flight ids, rotated Q) reuses a
    pool that is already in that state instead of building one."""
    from paper_2511_20426_amd.runner import CascadePool
    dev = torch.device("cuda:0")
    L, H, D, C = w.block_tokens, w.heads, w.head_dim, w.n_inflight
    if prepared is None:
        pool = CascadePool.for_workload(w, device=dev)
        gen = torch.Generator(device=dev).manual_seed(w.seed + 1)
        draw = lambda n: (torch.randn((n, H, D), generator=gen, device=dev) * w.input_scale).to(torch.bfloat16)
        kb, vb = [draw(L) for _ in range(C)], [draw(L) for _ in range(C)]
        for g in range(w.n_cached):
            pool.append(g, 0, 0, kb[g % C], vb[g % C])
            pool.ctx.kv_cache_promote(g)
        infl = list(range(w.n_cached, w.n_cached + C))
        pool.append_batch(infl, list(W.TIMESTEPS[::-1][:C]), 0, kb, vb)
        q_rot = pool.rope(draw(C * L), w.frames_per_block * infl[0])
    else:
        pool, infl, q_rot = prepared
    out = torch.empty_like(q_rot)
    res = {}
    cases = [(m, None) for m in modes] + [(m, s) for m in modes for s in shares]
    for mode, share in cases:
        def run():
            if share is None:
                pool.forward(q_rot, infl, mode, out=out)
            else:
                pool.forward(q_rot[:L], infl, mode, out=out[:L], share=(share, 1))
        run(); run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(launches):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / launches
        causal = mode == B.CA_BLOCK_CAUSAL
        if share is None:
            flops = w.flops(block_causal=causal)
        else:
            flops = 4.0 * D * L * (w.n_cached + (share + 1 if causal else C)) * L * H
        label = ("block_causal" if causal else "bidirectional") + ("" if share is None else f", share of block {share}")
        res[label] = {"ms": ms, "TFLOP/s": flops / ms / 1e9, "frac": flops / ms / 1e9 / PEAK_BF16_TFLOPS}
    return res


def time_layer_iteration(torch, W, w, iterations=4):
    """One steady-state cascade iteration of a whole self-attention layer at the workload's shape
    (model width = heads x head_dim, synthetic weights): QKV projection, K/V published, cascaded
    attention, output projection, then promote / evict / move on.  Two forms: five launches
    (projection, cache write, Q rotation, attention, projection) and three (the projection's
    epilogue publishes K/V, the attention kernel rotates Q)."""
    from paper_2511_20426_amd.runner import CascadePool, attention_layer
    dev = torch.device("cuda:0")
    L, H, D, C = w.block_tokens, w.heads, w.head_dim, w.n_inflight
    width = H * D
    gen = torch.Generator(device=dev).manual_seed(3)
    x = torch.randn((C * L, width), generator=gen, device=dev).to(torch.bfloat16)
    w_qkv = (torch.randn((3 * width, width), generator=gen, device=dev) / width ** 0.5).to(torch.bfloat16)
    w_out = (torch.randn((width, width), generator=gen, device=dev) / width ** 0.5).to(torch.bfloat16)
    res = {}
    for label, kw in (("five_launches", dict(rotate_q_in_kernel=False, publish_in_projection=False)),
                      ("three_launches", dict(rotate_q_in_kernel=True, publish_in_projection=True))):
        pool = CascadePool.for_workload(w, device=dev)
        for g in range(w.n_cached):                       # the clean window: blocks that ran alone
            attention_layer(pool, x[:L], w_qkv, w_out, [g], [0], 0, 0, **kw)
            pool.ctx.kv_cache_promote(g)
        b = w.n_cached
        ev = []
        for it in range(iterations + 1):                  # the first iteration warms up
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            attention_layer(pool, x, w_qkv, w_out, list(range(b, b + C)), list(W.TIMESTEPS[::-1][:C]), 0, 0, **kw)
            pool.ctx.kv_cache_promote(b)
            pool.ctx.kv_cache_evict(b - w.n_cached)
            e1.record()
            b += 1
            ev.append((e0, e1))
        torch.cuda.synchronize()
        ms = sum(a.elapsed_time(c) for a, c in ev[1:]) / iterations
        flops = w.flops() + 2.0 * C * L * width * (3 * width) + 2.0 * C * L * width * width
        res[label] = {"ms": ms, "TFLOP/s": flops / ms / 1e9, "frac": flops / ms / 1e9 / PEAK_BF16_TFLOPS}
        del pool
    return res


def time_qkv_projection(torch, W, w, launches=10):
    """The QKV projection of the blocks in flight at the workload's shape (model width = heads x
    head_dim), three ways: layer_linear_bf16 alone, kv_cache_append_batch on its k and v columns,
    and layer_qkv_publish, which does both in one launch."""
    from paper_2511_20426_amd.runner import CascadePool, linear
    dev = torch.device("cuda:0")
    L, H, D, C = w.block_tokens, w.heads, w.head_dim, w.n_inflight
    width, n = H * D, C * L
    gen = torch.Generator(device=dev).manual_seed(5)
    x = torch.randn((n, width), generator=gen, device=dev).to(torch.bfloat16)
    w_qkv = (torch.randn((3 * width, width), generator=gen, device=dev) / width ** 0.5).to(torch.bfloat16)
    pool = CascadePool.for_workload(w, device=dev)
    qkv = torch.empty((n, 3, H, D), dtype=torch.bfloat16, device=dev)
    q = torch.empty((n, H, D), dtype=torch.bfloat16, device=dev)
    ids, ts = list(range(w.n_cached, w.n_cached + C)), list(W.TIMESTEPS[::-1][:C])
    ks, vs = [qkv[i * L:(i + 1) * L, 1] for i in range(C)], [qkv[i * L:(i + 1) * L, 2] for i in range(C)]
    cases = (("layer_linear_bf16", lambda: linear(x, w_qkv, out=qkv.view(n, 3 * width))),
             ("kv_cache_append_batch", lambda: pool.append_batch(ids, ts, 0, ks, vs)),
             ("layer_qkv_publish", lambda: pool.qkv_publish(x, w_qkv, ids, ts, 0, q_out=q)))
    res = {}
    for label, run in cases:
        run(); run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(launches):
            run()
        e1.record()
        torch.cuda.synchronize()
        res[label] = {"ms": e0.elapsed_time(e1) / launches}
    flops = 2.0 * n * 3 * width * width
    for label in ("layer_linear_bf16", "layer_qkv_publish"):
        res[label]["TFLOP/s"] = flops / res[label]["ms"] / 1e9
        res[label]["frac"] = res[label]["TFLOP/s"] / PEAK_BF16_TFLOPS
    return res


def time_streaming_protocol(torch, W, B, w, blocks=13):
    """The paper's streaming protocol (Sec. 4: rate over the 8th and 9th block of a 13-block
    rollout) for one attention layer at the workload's shape, driven by the library's scheduler
    (Alg. 1): cold start, ramp-up, steady state, drain; one untimed pass first."""
    from paper_2511_20426_amd.runner import CascadePool
    from paper_2511_20426_amd.rollout import CascadeRollout, streaming_rate
    dev = torch.device("cuda:0")
    L, H, D = w.block_tokens, w.heads, w.head_dim
    gen = torch.Generator(device=dev).manual_seed(w.seed)
    bank = [tuple((torch.randn((L, H, D), generator=gen, device=dev) * w.input_scale).to(torch.bfloat16)
                  for _ in range(3)) for _ in range(len(W.TIMESTEPS))]
    out = {}
    for rep in range(2):
        pool = CascadePool.for_workload(w, device=dev)
        ro = CascadeRollout(pool, blocks, W.TIMESTEPS, lambda g, ti, it, i: bank[i], mode=B.CA_BIDIRECTIONAL, timed=True)
        recs = ro.run()
        if rep:
            out = {"iterations_per_s": streaming_rate(recs), "iteration_ms": [r.ms for r in recs if r.emitted in (7, 8)],
                   "blocks_per_s_whole_rollout": blocks / (sum(r.ms for r in recs) * 1e-3), "iterations": len(recs)}
        del ro, pool
    # the cascade types as schedules (Fig. 7: block j enters `lag` iterations after block j-1; lag 5, 3, 2, 1
    # keep 1, 2, 3, 5 blocks in flight): the whole 13-block rollout, ramp-up and drain included
    out["cascade_types"] = {}
    for lag, name in ((5, "P1"), (3, "P2"), (2, "P3"), (1, "P4")):
        pool = CascadePool.for_workload(w, device=dev)
        ro = CascadeRollout(pool, blocks, W.TIMESTEPS, lambda g, ti, it, i: bank[i], mode=B.CA_BIDIRECTIONAL, timed=True, lag=lag)
        recs = ro.run()
        out["cascade_types"][name] = {"lag": lag, "iterations": len(recs), "blocks_per_s": blocks / (sum(r.ms for r in recs) * 1e-3)}
        del ro, pool
    return out


# The projections either side of the attention at the Wan-14B width for five blocks in flight
# (not part of the default step: --workload linear_qkv_14b / linear_out_14b)
LINEAR_WORKLOADS = {"linear_qkv_14b": (23400, 15360, 5120), "linear_out_14b": (23400, 5120, 5120)}


def bench_linear(args, torch, W, B) -> int:
    from paper_2511_20426_amd.runner import linear
    import numpy as np
    M, N, K = LINEAR_WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev).manual_seed(0)
    x = torch.randn((M, K), generator=gen, device=dev).to(torch.bfloat16)
    wt = (torch.randn((N, K), generator=gen, device=dev) / K ** 0.5).to(torch.bfloat16)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    for _ in range(args.warmup):
        linear(x, wt, out=y)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        linear(x, wt, out=y)
    e1.record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    kms = e0.elapsed_time(e1) / args.steps
    flops = 2.0 * M * N * K
    result = {
        "metric": "bf16 linear (y = x w^T) TFLOP/s, Wan-14B width, 5 blocks of tokens", "value": flops / ms / 1e9,
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "m_rows": M, "n_out": N, "k_in": K, "flops_per_step": flops},
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_kernel", "achieved": flops / kms / 1e9,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": flops / kms / 1e9 / PEAK_BF16_TFLOPS,
                     "avg_launch_ms": kms, "traffic": None},
    }
    if not args.no_cpu_baseline:
        from oracle import cascade_oracle as orc
        rows = 512
        xs = W.to_f64(W.f32_to_bf16_bits(x[:rows].float().cpu().numpy()))
        ws = W.to_f64(W.f32_to_bf16_bits(wt.float().cpu().numpy()))
        t0, n = time.perf_counter(), 0
        while time.perf_counter() - t0 < 10.0:
            orc.layer_linear(xs, ws)
            n += 1
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        result["cpu_baseline"] = {"value": 2.0 * rows * N * K * n / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores),
                                  "kind": "oracle", "sample": f"fp64 numpy oracle on the first {rows} rows, {n} passes in {dt:.1f} s"}
    print(json.dumps(result))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4_wan14b_cascade5")
    ap.add_argument("--mode", default="bidirectional", choices=["bidirectional", "block_causal"])
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--inflight", type=int, default=None,
                    help="blocks in flight (cascade types P1..P4 of Fig. 7: 1, 2, 3, 5); default: the workload's")
    ap.add_argument("--cached", type=int, default=None,
                    help="clean cached blocks (2 = the paper's 7-block window accounting); default: the workload's")
    ap.add_argument("--share", type=int, default=None,
                    help="time one device's share of the step under the paper's temporal parallelism (one "
                         "in-flight block per GPU, every GPU holding the whole pool): only the queries of "
                         "in-flight block SHARE (0 = oldest) are rotated and attended; the five appends stand "
                         "in for the K/V exchange")
    ap.add_argument("--two-launch-q", action="store_true",
                    help="rotate Q with rope3d_apply and attend with cascade_attn_forward (two launches, Q makes a "
                         "round trip through HBM) instead of cascade_attn_forward_rope")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the attention-only timings of the other shapes and modes")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy instead (known traffic, for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        return 2

    import torch
    import workloads as W
    from paper_2511_20426_amd import binding as B
    from paper_2511_20426_amd.runner import CascadePool

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    if args.copy_calibration:
        x = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda:0")      # 1 GiB read + 1 GiB written
        y = torch.empty_like(x)
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": x.numel() * 2, "copy_bytes_written": x.numel() * 2}))
        return 0
    if args.workload in LINEAR_WORKLOADS:
        return bench_linear(args, torch, W, B)
    w = W.CONFIGS[args.workload]
    if args.inflight is not None or args.cached is not None:
        from dataclasses import replace
        ni = w.n_inflight if args.inflight is None else args.inflight
        nc = w.n_cached if args.cached is None else args.cached
        if not (1 <= ni <= w.max_inflight and 1 <= nc <= w.window_blocks):
            print("--inflight must be in 1..%d and --cached in 1..%d" % (w.max_inflight, w.window_blocks),
                  file=sys.stderr)
            return 2
        if (ni, nc) != (w.n_inflight, w.n_cached):
            w = replace(w, name="%s[inflight=%d,cached=%d]" % (w.name, ni, nc), n_inflight=ni, n_cached=nc)
    mode = B.CA_BIDIRECTIONAL if args.mode == "bidirectional" else B.CA_BLOCK_CAUSAL
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    L, H, D, C = w.block_tokens, w.heads, w.head_dim, w.n_inflight
    pool = CascadePool.for_workload(w, device=dev)
    pool.ctx.set_kernel_variant(args.variant)
    gen = torch.Generator(device=dev).manual_seed(w.seed)
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32

    def draw(n):
        return (torch.randn((n, H, D), generator=gen, device=dev, dtype=torch.float32) * w.input_scale).to(dt)

    if args.share is not None and not 0 <= args.share < C:
        print("--share must be in 0..%d" % (C - 1), file=sys.stderr)
        return 2
    q = draw(C * L)
    k_blocks = [draw(L) for _ in range(C)]
    v_blocks = [draw(L) for _ in range(C)]
    q_rot = torch.empty_like(q)
    out = torch.empty_like(q)

    # steady-state start: n_cached clean blocks 0..n_cached-1
    for g in range(w.n_cached):
        pool.append(g, 0, 0, k_blocks[g % C], v_blocks[g % C])
        pool.ctx.kv_cache_promote(g)
    timesteps = list(W.TIMESTEPS[::-1])            # oldest in-flight block is the cleanest (Alg. 1)
    state = {"b": w.n_cached}
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    ev_a = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]

    fused_q = args.share is None and not args.two_launch_q and w.dtype == "bf16"

    def step(i_timed=None):
        b = state["b"]
        infl = list(range(b, b + C))
        if i_timed is not None:
            ev_a[i_timed][0].record()
        pool.append_batch(infl, timesteps[:C], 0, k_blocks, v_blocks)   # a1: publish K/V, one launch
        if i_timed is not None:
            ev_a[i_timed][1].record()
        if fused_q:
            pass                                                       # a2 happens inside the attention kernel
        elif args.share is None:
            pool.rope(q, w.frames_per_block * b, out=q_rot)            # a2
        else:
            pool.rope(q[:L], w.frames_per_block * (b + args.share), out=q_rot[:L])
        if i_timed is not None:
            ev_a[i_timed][2].record()
            ev[i_timed][0].record()
        if fused_q:
            pool.forward_rope(q, infl, mode, out=out)                  # a2-a6
        elif args.share is None:
            pool.forward(q_rot, infl, mode, out=out)                   # a3-a6
        else:
            pool.forward(q_rot[:L], infl, mode, out=out[:L], share=(args.share, 1))
        if i_timed is not None:
            ev[i_timed][1].record()
        pool.ctx.kv_cache_promote(b)                                   # a7
        pool.ctx.kv_cache_evict(b - w.n_cached)
        state["b"] = b + 1

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt_s = time.perf_counter() - t0

    flops = w.flops(block_causal=(mode == B.CA_BLOCK_CAUSAL))
    n_rot = C
    if args.share is not None:
        vis_blocks = w.n_cached + (args.share + 1 if mode == B.CA_BLOCK_CAUSAL else C)
        flops = 4.0 * D * L * vis_blocks * L * H
        n_rot = 1
    ms_per_step = dt_s / args.steps * 1e3
    attn_ms = sum(a.elapsed_time(b) for a, b in ev) / args.steps
    achieved = flops / (attn_ms * 1e-3) / 1e12
    result = {
        "metric": "cascaded-attn TFLOP/s + % bf16 MFMA peak, Wan-14B shape, 5 in-flight blocks" +
                  ("" if args.share is None else ", one device's share (queries of in-flight block %d)" % args.share),
        "value": flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "pct_of_bf16_mfma_peak": 100.0 * flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "heads": H, "head_dim": D, "tokens_per_block": L,
                   "inflight_blocks": C, "cached_blocks": w.n_cached, "mode": args.mode,
                   "n_q": n_rot * L, "n_kv": (w.n_cached + C) * L, "flops_per_step": flops,
                   "step": "kv_cache_append_batch(%d blocks) + %s + promote/evict"
                           % (C, "cascade_attn_forward_rope (Q rotated inside the attention kernel)" if fused_q else
                              "rope3d_apply(Q) + " + ("cascade_attn_forward" if args.share is None
                                                      else "cascade_attn_forward_share"))},
        "roofline": {"bound": "mfma", "kernel": "attn_bf16_kernel<true>" if fused_q else "attn_bf16_kernel<false>", "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "avg_launch_ms": attn_ms,
                     "traffic": ATTN_TRAFFIC_BYTES_C4 if (w.name == "c4_wan14b_cascade5" and
                                                          mode == B.CA_BIDIRECTIONAL and
                                                          args.share is None) else None,
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this "
                                       "command (profiles/c4_wan14b_cascade5_hbm_traffic.txt), not measured in this run"},
    }
    # the two HBM-bound steps: every element read once and written once
    eb = 2 if w.dtype == "bf16" else 4
    append_ms = sum(e[0].elapsed_time(e[1]) for e in ev_a) / args.steps / C
    if fused_q:                                   # a2 as its own kernel, outside the step: five launches
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        pool.rope(q, w.frames_per_block * state["b"], out=q_rot)
        e0.record()
        for _ in range(5):
            pool.rope(q, w.frames_per_block * state["b"], out=q_rot)
        e1.record()
        torch.cuda.synchronize()
        rope_ms = e0.elapsed_time(e1) / 5
    else:
        rope_ms = sum(e[1].elapsed_time(e[2]) for e in ev_a) / args.steps
    append_gbs = 2 * (2 * L * H * D * eb) / (append_ms * 1e-3) / 1e9
    rope_gbs = 2 * (n_rot * L * H * D * eb) / (rope_ms * 1e-3) / 1e9
    result["secondary"] = {
        "kv_cache_append": {"us_per_block": append_ms * 1e3, "GB/s": append_gbs, "frac_of_hbm_peak": append_gbs / PEAK_HBM_GBS},
        "rope3d_apply": {"us": rope_ms * 1e3, "GB/s": rope_gbs, "frac_of_hbm_peak": rope_gbs / PEAK_HBM_GBS,
                         "in_step": not fused_q}}
    # what the matrix pipes sustain on this machine with nothing else in the loop (the nominal peak
    # assumes 2.4 GHz; under a full MFMA load with toggling operands the chip clocks lower)
    probe = torch.empty(1 << 16, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    rnd = B.mfma_microbench(1, 100000, probe.data_ptr(), probe.numel(), stream)
    zer = B.mfma_microbench(0, 100000, probe.data_ptr(), probe.numel(), stream)
    result["roofline"]["mfma_only_microbench"] = {
        "random_operands": {"TFLOP/s": rnd[0], "clock_GHz": rnd[1]},
        "zero_operands": {"TFLOP/s": zer[0], "clock_GHz": zer[1]},
        "achieved_over_random_operands": achieved / rnd[0]}
    # The other shapes and modes of the method, attention launch alone (events, a few launches
    # each): the headline workload in block-causal mode (Sec. 4.2) and as one device's share under
    # the paper's temporal parallelism (Sec. 3.3), the Wan-1.3B cascade in both modes, and the
    # sequential one-block baseline (cascade type P1 of Fig. 7).
    if (w.name == "c4_wan14b_cascade5" and mode == B.CA_BIDIRECTIONAL and args.share is None
            and not args.no_secondary):
        both = (B.CA_BIDIRECTIONAL, B.CA_BLOCK_CAUSAL)
        infl = list(range(state["b"], state["b"] + C))              # the next iteration's blocks, published
        pool.append_batch(infl, timesteps[:C], 0, k_blocks, v_blocks)
        pool.rope(q, w.frames_per_block * infl[0], out=q_rot)
        result["secondary"]["attention_only"] = {
            "c4_wan14b_cascade5": time_attention_only(torch, W, B, w, both, shares=(0, C - 1), prepared=(pool, infl, q_rot)),
            "c3_wan1p3b_cascade5": time_attention_only(torch, W, B, W.CONFIGS["c3_wan1p3b_cascade5"], both),
            "c2_wan1p3b_seq": time_attention_only(torch, W, B, W.CONFIGS["c2_wan1p3b_seq"], (B.CA_BIDIRECTIONAL,)),
        }
        # cascade types P1..P4 (Fig. 7: 1, 2, 3, 5 blocks in flight) at the 14B shape, on the 6-block
        # clean window of the headline and on the paper's own window accounting (7 blocks = 5 in
        # flight + 2 cached, Sec. 4)
        from dataclasses import replace
        sweep = {}
        for nc in (6, 2):
            for ni in (1, 2, 3, 5):
                if (ni, nc) == (w.n_inflight, w.n_cached):
                    continue                                            # the headline itself
                wv = replace(w, name=f"{w.name}[inflight={ni},cached={nc}]", n_inflight=ni, n_cached=nc)
                sweep[f"inflight={ni},cached={nc}"] = time_attention_only(torch, W, B, wv, (B.CA_BIDIRECTIONAL,))["bidirectional"]
        result["secondary"]["attention_only"]["cascade_types_14b"] = sweep
        del pool
        result["secondary"]["layer_iteration_14b"] = time_layer_iteration(torch, W, w)
        result["secondary"]["qkv_projection_14b"] = time_qkv_projection(torch, W, w)
        result["secondary"]["streaming_protocol_14b"] = time_streaming_protocol(torch, W, B, w)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
