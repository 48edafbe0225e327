"""Torch plumbing around the C ABI: device memory for the pool and the current HIP stream.

No arithmetic of the method happens here; every tensor handed to the library is passed as a
raw device address.
"""
from __future__ import annotations

from typing import Sequence

import torch

from . import binding as B


def torch_dtype(dtype: str):
    return {"bf16": torch.bfloat16, "f32": torch.float32}[dtype]


class CascadePool:
    """A ca_ctx over a pool tensor allocated with torch on the current device."""

    def __init__(self, *, heads, head_dim, frames_per_block, grid_h, grid_w, rope_dims, rope_theta,
                 sink_blocks, window_blocks, max_inflight, page_tokens, dtype, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("CascadePool needs a GPU; use binding.Context(cfg) for metadata-only work")
        self.dtype = dtype
        self.device = torch.device(device)
        self.cfg = B.make_config(heads=heads, head_dim=head_dim, frames_per_block=frames_per_block,
                                 grid_h=grid_h, grid_w=grid_w, rope_dims=rope_dims, rope_theta=rope_theta,
                                 sink_blocks=sink_blocks, window_blocks=window_blocks,
                                 max_inflight=max_inflight, page_tokens=page_tokens, dtype=dtype)
        nbytes = B.pool_bytes(self.cfg)
        if nbytes == 0:
            raise ValueError("configuration rejected by ca_pool_bytes")
        self.pool = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.ctx = B.Context(self.cfg, self.pool.data_ptr(), nbytes)
        self.block_tokens = frames_per_block * grid_h * grid_w
        self.frames_per_block = frames_per_block
        self.heads, self.head_dim = heads, head_dim

    @classmethod
    def for_workload(cls, w, device="cuda:0"):
        return cls(heads=w.heads, head_dim=w.head_dim, frames_per_block=w.frames_per_block,
                   grid_h=w.grid_h, grid_w=w.grid_w, rope_dims=w.rope_dims, rope_theta=w.rope_theta,
                   sink_blocks=w.sink_blocks, window_blocks=max(w.window_blocks, w.n_cached - w.sink_blocks),
                   max_inflight=w.max_inflight, page_tokens=w.page_tokens, dtype=w.dtype, device=device)

    def _stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def _check(self, t: torch.Tensor) -> None:
        assert t.is_cuda and t.dtype == torch_dtype(self.dtype) and t.dim() == 3 and t.stride(2) == 1
        assert t.shape[1] == self.heads and t.shape[2] == self.head_dim

    def append(self, block_id: int, timestep: int, epoch: int, k: torch.Tensor, v: torch.Tensor) -> int:
        self._check(k); self._check(v)
        assert k.shape[0] == self.block_tokens and k.stride() == v.stride() and k.shape == v.shape
        return self.ctx.kv_cache_append(block_id, timestep, epoch, k.data_ptr(), v.data_ptr(),
                                        k.stride(0), k.stride(1), self._stream())

    def append_batch(self, block_ids: Sequence[int], timesteps: Sequence[int], epoch: int,
                     ks: Sequence[torch.Tensor], vs: Sequence[torch.Tensor]) -> list[int]:
        """All blocks of one cascade iteration in one launch; the tensors share their strides."""
        for k, v in zip(ks, vs):
            self._check(k); self._check(v)
            assert k.shape[0] == self.block_tokens and k.shape == v.shape
            assert k.stride() == ks[0].stride() and v.stride() == ks[0].stride()
        return self.ctx.kv_cache_append_batch(list(block_ids), list(timesteps), epoch,
                                              [k.data_ptr() for k in ks], [v.data_ptr() for v in vs],
                                              ks[0].stride(0), ks[0].stride(1), self._stream())

    def rope(self, x: torch.Tensor, first_frame: int, out: torch.Tensor | None = None) -> torch.Tensor:
        """Rotate x [n, H, D] (any token / head strides) into `out` (its own strides; default: a new
        contiguous tensor).  x is out is allowed."""
        self._check(x)
        y = torch.empty(x.shape, dtype=x.dtype, device=x.device) if out is None else out
        self._check(y)
        assert y.shape == x.shape
        self.ctx.rope3d_apply_strided(x.data_ptr(), x.stride(0), x.stride(1), y.data_ptr(), y.stride(0), y.stride(1),
                                      x.shape[0], first_frame, self._stream())
        return y

    def forward(self, q_rot: torch.Tensor, inflight: Sequence[int], mode: int,
                out: torch.Tensor | None = None, share: tuple[int, int] | None = None,
                static_scratch: bool = False) -> torch.Tensor:
        """Attention of the in-flight blocks' queries; with share = (first, count) only of blocks
        first .. first+count-1 of `inflight` (q_rot and the result then hold just those);
        static_scratch: through cascade_attn_forward_static (`out` must then be given: that call
        is for callers that do not allocate)."""
        self._check(q_rot)
        n_q = len(inflight) if share is None else share[1]
        assert q_rot.is_contiguous() and q_rot.shape[0] == n_q * self.block_tokens
        o = torch.empty_like(q_rot) if out is None else out
        assert o.is_contiguous() and o.shape == q_rot.shape
        if static_scratch:
            assert share is None and out is not None
            self.ctx.cascade_attn_forward_static(q_rot.data_ptr(), list(inflight), mode, o.data_ptr(), self._stream())
        elif share is None:
            self.ctx.cascade_attn_forward(q_rot.data_ptr(), list(inflight), mode, o.data_ptr(), self._stream())
        else:
            self.ctx.cascade_attn_forward_share(q_rot.data_ptr(), list(inflight), share[0], share[1], mode,
                                                o.data_ptr(), self._stream())
        return o


def _forward_rope(self, q_raw: torch.Tensor, inflight: Sequence[int], mode: int,
                  out: torch.Tensor | None = None) -> torch.Tensor:
    """Attention on queries that are not rotated yet (cascade_attn_forward_rope): q_raw [C*L, H, D]
    with any token / head strides; the result is a contiguous tensor of that shape."""
    self._check(q_raw)
    assert q_raw.shape[0] == len(inflight) * self.block_tokens
    o = torch.empty(q_raw.shape, dtype=q_raw.dtype, device=q_raw.device) if out is None else out
    assert o.is_contiguous() and o.shape == q_raw.shape
    self.ctx.cascade_attn_forward_rope(q_raw.data_ptr(), q_raw.stride(0), q_raw.stride(1), list(inflight), mode,
                                       o.data_ptr(), self._stream())
    return o


CascadePool.forward_rope = _forward_rope


def _qkv_publish(self, x: torch.Tensor, w_qkv: torch.Tensor, block_ids: Sequence[int], timesteps: Sequence[int],
                 epoch: int, q_out: torch.Tensor | None = None) -> torch.Tensor:
    """QKV projection of the blocks in flight with their K/V published to the pool by the same
    launch (layer_qkv_publish); returns the packed, unrotated queries [C*L, H, D]."""
    n = len(block_ids) * self.block_tokens
    width = self.heads * self.head_dim
    assert x.is_cuda and x.dtype == torch.bfloat16 and x.dim() == 2 and x.shape[0] == n and x.stride(1) == 1
    assert w_qkv.shape == (3 * width, x.shape[1]) and w_qkv.stride(1) == 1 and w_qkv.dtype == torch.bfloat16
    q = torch.empty((n, self.heads, self.head_dim), dtype=torch.bfloat16, device=x.device) if q_out is None else q_out
    assert q.is_contiguous() and q.shape == (n, self.heads, self.head_dim)
    self.ctx.layer_qkv_publish(list(block_ids), list(timesteps), epoch, x.data_ptr(), x.stride(0), w_qkv.data_ptr(),
                               w_qkv.stride(0), x.shape[1], q.data_ptr(), self._stream())
    return q


CascadePool.qkv_publish = _qkv_publish


def linear(x: torch.Tensor, w: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """y = x @ w.T through layer_linear_bf16: x [M, K], w [N, K], y [M, N], bf16, rows may be
    strided (last dimension contiguous)."""
    assert x.is_cuda and w.is_cuda and x.dtype == torch.bfloat16 and w.dtype == torch.bfloat16
    assert x.dim() == 2 and w.dim() == 2 and x.shape[1] == w.shape[1] and x.stride(1) == 1 and w.stride(1) == 1
    y = torch.empty((x.shape[0], w.shape[0]), dtype=torch.bfloat16, device=x.device) if out is None else out
    assert y.shape == (x.shape[0], w.shape[0]) and y.stride(1) == 1 and y.dtype == torch.bfloat16
    B.layer_linear_bf16(x.data_ptr(), w.data_ptr(), y.data_ptr(), x.shape[0], w.shape[0], x.shape[1],
                        x.stride(0), w.stride(0), y.stride(0), torch.cuda.current_stream(x.device).cuda_stream)
    return y


def attention_layer(pool: CascadePool, x: torch.Tensor, w_qkv: torch.Tensor, w_out: torch.Tensor,
                    inflight: Sequence[int], timesteps: Sequence[int], epoch: int, mode: int,
                    rotate_q_in_kernel: bool = True, publish_in_projection: bool = False) -> torch.Tensor:
    """One self-attention layer around the shared pool, for the blocks in flight (oldest first,
    consecutive in the video): QKV projection, K/V of every block published to the cache, Q
    rotated, cascaded attention, output projection.  x [C*L, width], w_qkv [3*width, width] with
    output rows ordered (q|k|v, head, dim), w_out [width, width]; width = heads * head_dim.
    Library calls only; the q/k/v handed on are strided views of the projection's output.  The
    queries go to the attention kernel as they are (it rotates them while loading), or, with
    rotate_q_in_kernel=False, through rope3d_apply into a contiguous tensor first.  With
    publish_in_projection the first two steps are one launch (layer_qkv_publish): K/V go from the
    projection's epilogue straight into pool pages; three launches per layer in all."""
    L, H, D = pool.block_tokens, pool.heads, pool.head_dim
    n = len(inflight) * L
    assert x.shape == (n, H * D) and w_qkv.shape == (3 * H * D, H * D) and w_out.shape == (H * D, H * D)
    if publish_in_projection:
        q = pool.qkv_publish(x, w_qkv, inflight, timesteps, epoch)
        o = pool.forward_rope(q, inflight, mode)
        return linear(o.view(n, H * D), w_out)
    qkv = linear(x, w_qkv).view(n, 3, H, D)
    blocks = [qkv[i * L:(i + 1) * L] for i in range(len(inflight))]
    pool.append_batch(inflight, timesteps, epoch, [b[:, 1] for b in blocks], [b[:, 2] for b in blocks])
    if rotate_q_in_kernel:
        o = pool.forward_rope(qkv[:, 0], inflight, mode)
    else:
        q_rot = pool.rope(qkv[:, 0], pool.frames_per_block * inflight[0])     # strided view -> contiguous
        o = pool.forward(q_rot, inflight, mode)
    return linear(o.view(n, H * D), w_out)
