"""ctypes binding of libcascade_attn.so (include/cascade_attn.h).

Argument marshalling only: every step of the path (rotary embedding, cache write,
attention) runs in the library's HIP kernels.  Device buffers are passed as raw
addresses (e.g. torch.Tensor.data_ptr()), the stream as a raw hipStream_t
(torch.cuda.current_stream().cuda_stream).  There is no CPU fallback: if the
library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CASCADE_ATTN_LIB") or os.path.join(_PKG, "libcascade_attn.so")

CA_OK, CA_EINVAL, CA_ENOSPC, CA_ENOENT, CA_ESTATE, CA_EUNSUPPORTED, CA_ENOPOOL, CA_EDEVICE, CA_ETOOBIG = (
    0, -1, -2, -3, -4, -5, -6, -7, -8)
CA_F32, CA_BF16 = 0, 1
CA_BIDIRECTIONAL, CA_BLOCK_CAUSAL = 0, 1
CA_FREE, CA_NOISY, CA_CLEAN, CA_SINK = 0, 1, 2, 3

# every symbol include/cascade_attn.h declares
EXPORTS = (
    "ca_pool_bytes", "ca_create", "ca_destroy", "kv_cache_append", "kv_cache_append_batch", "kv_cache_promote",
    "kv_cache_evict", "kv_cache_retag", "kv_cache_snapshot", "kv_cache_page_index",
    "rope3d_apply", "rope3d_apply_strided", "cascade_attn_forward", "cascade_attn_forward_share", "cascade_attn_forward_static", "cascade_attn_forward_rope", "ca_debug_visibility", "ca_set_kernel_variant",
    "ca_strerror", "ca_last_device_error",
    "ca_mfma_microbench", "layer_linear_bf16", "layer_qkv_publish",
    "ca_sched_create", "ca_sched_create_lagged", "ca_sched_destroy", "ca_sched_batch", "ca_sched_advance", "ca_sched_state",
)


class ca_config(C.Structure):
    _fields_ = [
        ("heads", C.c_int32), ("head_dim", C.c_int32),
        ("frames_per_block", C.c_int32), ("grid_h", C.c_int32), ("grid_w", C.c_int32),
        ("rope_dim_t", C.c_int32), ("rope_dim_h", C.c_int32), ("rope_dim_w", C.c_int32),
        ("rope_theta", C.c_double),
        ("sink_blocks", C.c_int32), ("window_blocks", C.c_int32), ("max_inflight", C.c_int32),
        ("page_tokens", C.c_int32), ("dtype", C.c_int32),
    ]


class ca_slot_info(C.Structure):
    _fields_ = [("slot", C.c_int32), ("state", C.c_int32), ("block_id", C.c_int64),
                ("timestep", C.c_int32), ("prompt_epoch", C.c_int32)]


class ca_sched_entry(C.Structure):
    _fields_ = [("block_id", C.c_int64), ("timestep_index", C.c_int32), ("timestep", C.c_int32)]


class CascadeAttnError(RuntimeError):
    def __init__(self, code: int, what: str):
        detail = lib.ca_last_device_error().decode() if code == CA_EDEVICE else ""
        super().__init__(f"{what}: {strerror(code)} ({code}) {detail}")
        self.code = code


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH) and "CASCADE_ATTN_LIB" not in os.environ:
        # nothing built yet (a fresh checkout): build once, in-tree; there is no other path
        import importlib.util
        spec = importlib.util.spec_from_file_location(
            "_cascade_attn_build", os.path.join(os.path.dirname(os.path.abspath(__file__)), "_build.py"))
        builder = importlib.util.module_from_spec(spec)
        try:
            spec.loader.exec_module(builder)
            builder.build()
        except Exception as e:  # no hipcc, compile error, ...
            raise ImportError(f"{LIB_PATH} is missing and could not be built: {e}") from e
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    # One HIP runtime per process: torch ships its own libamdhip64.  Importing torch first
    # makes the loader resolve this library's libamdhip64 dependency to the copy torch has
    # already loaded, so the tensors torch allocates and our launches share one runtime.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.ca_pool_bytes.restype = C.c_size_t
    lib.ca_pool_bytes.argtypes = [C.POINTER(ca_config)]
    lib.ca_create.restype = i32
    lib.ca_create.argtypes = [C.POINTER(ca_config), vp, C.c_size_t, C.POINTER(vp)]
    lib.ca_destroy.restype = i32
    lib.ca_destroy.argtypes = [vp]
    lib.kv_cache_append.restype = i32
    lib.kv_cache_append.argtypes = [vp, i64, i32, i32, vp, vp, i64, i64, vp, C.POINTER(i32)]
    lib.kv_cache_promote.restype = i32
    lib.kv_cache_promote.argtypes = [vp, i64]
    lib.kv_cache_append_batch.restype = i32
    lib.kv_cache_append_batch.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(i32), i32, C.POINTER(vp), C.POINTER(vp),
                                          i64, i64, vp, C.POINTER(i32)]
    lib.kv_cache_evict.restype = i32
    lib.kv_cache_evict.argtypes = [vp, i64]
    lib.kv_cache_retag.restype = i32
    lib.kv_cache_retag.argtypes = [vp, i32]
    lib.kv_cache_snapshot.restype = i32
    lib.kv_cache_snapshot.argtypes = [vp, C.POINTER(ca_slot_info), i32, C.POINTER(i32)]
    lib.kv_cache_page_index.restype = i32
    lib.kv_cache_page_index.argtypes = [vp, i64, i32, i32, C.POINTER(i64)]
    lib.rope3d_apply.restype = i32
    lib.rope3d_apply.argtypes = [vp, vp, vp, i64, i64, i64, i64, vp]
    lib.rope3d_apply_strided.restype = i32
    lib.rope3d_apply_strided.argtypes = [vp, vp, i64, i64, vp, i64, i64, i64, i64, vp]
    lib.cascade_attn_forward.restype = i32
    lib.cascade_attn_forward.argtypes = [vp, vp, C.POINTER(i64), i32, i32, vp, vp]
    lib.cascade_attn_forward_static.restype = i32
    lib.cascade_attn_forward_static.argtypes = [vp, vp, C.POINTER(i64), i32, i32, vp, vp]
    lib.cascade_attn_forward_rope.restype = i32
    lib.cascade_attn_forward_rope.argtypes = [vp, vp, i64, i64, C.POINTER(i64), i32, i32, vp, vp]
    lib.cascade_attn_forward_share.restype = i32
    lib.cascade_attn_forward_share.argtypes = [vp, vp, C.POINTER(i64), i32, i32, i32, i32, vp, vp]
    lib.ca_debug_visibility.restype = i32
    lib.ca_debug_visibility.argtypes = [vp, C.POINTER(i64), i32, i32, C.POINTER(C.c_uint8),
                                        C.POINTER(i64), i32, C.POINTER(i32)]
    lib.ca_set_kernel_variant.restype = i32
    lib.ca_set_kernel_variant.argtypes = [vp, i32]
    lib.ca_mfma_microbench.restype = i32
    lib.ca_mfma_microbench.argtypes = [i32, i32, vp, C.c_size_t, vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.layer_linear_bf16.restype = i32
    lib.layer_linear_bf16.argtypes = [vp, vp, vp, i64, i32, i32, i64, i64, i64, vp]
    lib.layer_qkv_publish.restype = i32
    lib.layer_qkv_publish.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(i32), i32, vp, i64, vp, i64, i32, vp, vp,
                                      C.POINTER(i32)]
    lib.ca_sched_create.restype = i32
    lib.ca_sched_create.argtypes = [i64, i32, C.POINTER(i32), i32, C.POINTER(vp)]
    lib.ca_sched_create_lagged.restype = i32
    lib.ca_sched_create_lagged.argtypes = [i64, C.POINTER(i32), i32, i32, C.POINTER(vp)]
    lib.ca_sched_destroy.restype = i32
    lib.ca_sched_destroy.argtypes = [vp]
    lib.ca_sched_batch.restype = i32
    lib.ca_sched_batch.argtypes = [vp, C.POINTER(ca_sched_entry), i32, C.POINTER(i32)]
    lib.ca_sched_advance.restype = i32
    lib.ca_sched_advance.argtypes = [vp, C.POINTER(i64), C.POINTER(i64)]
    lib.ca_sched_state.restype = i32
    lib.ca_sched_state.argtypes = [vp, C.POINTER(i64), C.POINTER(i32), C.POINTER(i32), C.POINTER(i64)]
    lib.ca_strerror.restype = C.c_char_p
    lib.ca_strerror.argtypes = [i32]
    lib.ca_last_device_error.restype = C.c_char_p
    lib.ca_last_device_error.argtypes = []
    return lib


lib = _load()


def strerror(code: int) -> str:
    return lib.ca_strerror(code).decode()


def _check(code: int, what: str) -> None:
    if code != CA_OK:
        raise CascadeAttnError(code, what)


def make_config(*, heads, head_dim, frames_per_block, grid_h, grid_w, rope_dims, rope_theta,
                sink_blocks, window_blocks, max_inflight, page_tokens, dtype) -> ca_config:
    dt = {"f32": CA_F32, "bf16": CA_BF16}.get(dtype, dtype)
    return ca_config(heads, head_dim, frames_per_block, grid_h, grid_w, rope_dims[0], rope_dims[1],
                     rope_dims[2], float(rope_theta), sink_blocks, window_blocks, max_inflight,
                     page_tokens, dt)


def pool_bytes(cfg: ca_config) -> int:
    return int(lib.ca_pool_bytes(C.byref(cfg)))


@dataclass
class SlotInfo:
    slot: int
    block_id: int
    state: int
    timestep: int
    prompt_epoch: int

    def astuple(self) -> Tuple[int, int, int, int, int]:
        return (self.slot, self.block_id, self.state, self.timestep, self.prompt_epoch)


class Context:
    """Thin owner of a ca_ctx*.  pool_ptr = 0 makes a metadata-only context."""

    def __init__(self, cfg: ca_config, pool_ptr: int = 0, pool_nbytes: int = 0):
        self.cfg = cfg
        h = C.c_void_p()
        _check(lib.ca_create(C.byref(cfg), C.c_void_p(pool_ptr or None), pool_nbytes, C.byref(h)),
               "ca_create")
        self._h = h

    def close(self) -> None:
        if self._h:
            lib.ca_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # cache
    def kv_cache_append(self, block_id: int, timestep: int, prompt_epoch: int, k_ptr: int, v_ptr: int,
                        tok_stride: int, head_stride: int, stream: int = 0) -> int:
        slot = C.c_int32(-1)
        _check(lib.kv_cache_append(self._h, block_id, timestep, prompt_epoch, C.c_void_p(k_ptr or None),
                                   C.c_void_p(v_ptr or None), tok_stride, head_stride,
                                   C.c_void_p(stream or None), C.byref(slot)), "kv_cache_append")
        return slot.value

    def kv_cache_append_batch(self, block_ids: Sequence[int], timesteps: Sequence[int], prompt_epoch: int,
                              k_ptrs: Sequence[int], v_ptrs: Sequence[int], tok_stride: int, head_stride: int,
                              stream: int = 0) -> List[int]:
        n = len(block_ids)
        assert len(timesteps) == n and len(k_ptrs) == n and len(v_ptrs) == n
        ids = (C.c_int64 * n)(*block_ids)
        ts = (C.c_int32 * n)(*timesteps)
        kp = (C.c_void_p * n)(*[p or None for p in k_ptrs])
        vp = (C.c_void_p * n)(*[p or None for p in v_ptrs])
        slots = (C.c_int32 * max(n, 1))()
        _check(lib.kv_cache_append_batch(self._h, n, ids, ts, prompt_epoch, kp, vp, tok_stride, head_stride,
                                         C.c_void_p(stream or None), slots), "kv_cache_append_batch")
        return [int(slots[i]) for i in range(n)]

    def layer_qkv_publish(self, block_ids: Sequence[int], timesteps: Sequence[int], prompt_epoch: int, x_ptr: int,
                          ldx: int, w_ptr: int, ldw: int, k_in: int, q_out_ptr: int, stream: int = 0) -> List[int]:
        n = len(block_ids)
        assert len(timesteps) == n
        ids = (C.c_int64 * n)(*block_ids)
        ts = (C.c_int32 * n)(*timesteps)
        slots = (C.c_int32 * max(n, 1))()
        _check(lib.layer_qkv_publish(self._h, n, ids, ts, prompt_epoch, C.c_void_p(x_ptr or None), ldx,
                                     C.c_void_p(w_ptr or None), ldw, k_in, C.c_void_p(q_out_ptr or None),
                                     C.c_void_p(stream or None), slots), "layer_qkv_publish")
        return [int(slots[i]) for i in range(n)]

    def kv_cache_promote(self, block_id: int) -> None:
        _check(lib.kv_cache_promote(self._h, block_id), "kv_cache_promote")

    def kv_cache_evict(self, block_id: int) -> None:
        _check(lib.kv_cache_evict(self._h, block_id), "kv_cache_evict")

    def kv_cache_retag(self, new_prompt_epoch: int) -> None:
        _check(lib.kv_cache_retag(self._h, new_prompt_epoch), "kv_cache_retag")

    def kv_cache_snapshot(self) -> List[SlotInfo]:
        n = C.c_int32(0)
        _check(lib.kv_cache_snapshot(self._h, None, 0, C.byref(n)), "kv_cache_snapshot")
        buf = (ca_slot_info * max(n.value, 1))()
        _check(lib.kv_cache_snapshot(self._h, buf, n.value, C.byref(n)), "kv_cache_snapshot")
        return [SlotInfo(b.slot, b.block_id, b.state, b.timestep, b.prompt_epoch) for b in buf[:n.value]]

    def kv_cache_page_index(self, block_id: int, page: int, head: int) -> int:
        out = C.c_int64(-1)
        _check(lib.kv_cache_page_index(self._h, block_id, page, head, C.byref(out)), "kv_cache_page_index")
        return out.value

    # device work
    def rope3d_apply(self, x_ptr: int, y_ptr: int, n_tokens: int, first_frame: int, tok_stride: int,
                     head_stride: int, stream: int = 0) -> None:
        _check(lib.rope3d_apply(self._h, C.c_void_p(x_ptr or None), C.c_void_p(y_ptr or None), n_tokens,
                                first_frame, tok_stride, head_stride, C.c_void_p(stream or None)),
               "rope3d_apply")

    def rope3d_apply_strided(self, x_ptr: int, x_tok_stride: int, x_head_stride: int, y_ptr: int,
                             y_tok_stride: int, y_head_stride: int, n_tokens: int, first_frame: int,
                             stream: int = 0) -> None:
        _check(lib.rope3d_apply_strided(self._h, C.c_void_p(x_ptr or None), x_tok_stride, x_head_stride,
                                        C.c_void_p(y_ptr or None), y_tok_stride, y_head_stride, n_tokens,
                                        first_frame, C.c_void_p(stream or None)), "rope3d_apply_strided")

    def cascade_attn_forward(self, q_ptr: int, inflight_block_ids: Sequence[int], mode: int, out_ptr: int,
                             stream: int = 0) -> None:
        ids = (C.c_int64 * len(inflight_block_ids))(*inflight_block_ids)
        _check(lib.cascade_attn_forward(self._h, C.c_void_p(q_ptr or None), ids, len(inflight_block_ids),
                                        mode, C.c_void_p(out_ptr or None), C.c_void_p(stream or None)),
               "cascade_attn_forward")

    def cascade_attn_forward_static(self, q_ptr: int, inflight_block_ids: Sequence[int], mode: int, out_ptr: int,
                                    stream: int = 0) -> None:
        ids = (C.c_int64 * len(inflight_block_ids))(*inflight_block_ids)
        _check(lib.cascade_attn_forward_static(self._h, C.c_void_p(q_ptr or None), ids, len(inflight_block_ids),
                                               mode, C.c_void_p(out_ptr or None), C.c_void_p(stream or None)),
               "cascade_attn_forward_static")

    def cascade_attn_forward_rope(self, q_ptr: int, q_tok_stride: int, q_head_stride: int,
                                  inflight_block_ids: Sequence[int], mode: int, out_ptr: int, stream: int = 0) -> None:
        ids = (C.c_int64 * len(inflight_block_ids))(*inflight_block_ids)
        _check(lib.cascade_attn_forward_rope(self._h, C.c_void_p(q_ptr or None), q_tok_stride, q_head_stride, ids,
                                             len(inflight_block_ids), mode, C.c_void_p(out_ptr or None),
                                             C.c_void_p(stream or None)), "cascade_attn_forward_rope")

    def cascade_attn_forward_share(self, q_ptr: int, inflight_block_ids: Sequence[int], first: int, count: int,
                                   mode: int, out_ptr: int, stream: int = 0) -> None:
        ids = (C.c_int64 * len(inflight_block_ids))(*inflight_block_ids)
        _check(lib.cascade_attn_forward_share(self._h, C.c_void_p(q_ptr or None), ids, len(inflight_block_ids),
                                              first, count, mode, C.c_void_p(out_ptr or None),
                                              C.c_void_p(stream or None)), "cascade_attn_forward_share")

    def debug_visibility(self, inflight_block_ids: Sequence[int], mode: int):
        """(vis [n_inflight][n_kv] as nested lists, kv_block_ids)."""
        n = len(inflight_block_ids)
        cap = 64
        ids = (C.c_int64 * n)(*inflight_block_ids)
        vis = (C.c_uint8 * (n * cap))()
        kv = (C.c_int64 * cap)()
        n_kv = C.c_int32(0)
        _check(lib.ca_debug_visibility(self._h, ids, n, mode, vis, kv, cap, C.byref(n_kv)),
               "ca_debug_visibility")
        m = n_kv.value
        return [[int(vis[i * m + r]) for r in range(m)] for i in range(n)], [int(kv[r]) for r in range(m)]

    def set_kernel_variant(self, variant: int) -> None:
        _check(lib.ca_set_kernel_variant(self._h, variant), "ca_set_kernel_variant")


def layer_linear_bf16(x_ptr: int, w_ptr: int, y_ptr: int, m_rows: int, n_out: int, k_in: int,
                      ldx: int, ldw: int, ldy: int, stream: int = 0) -> None:
    _check(lib.layer_linear_bf16(x_ptr, w_ptr, y_ptr, m_rows, n_out, k_in, ldx, ldw, ldy, stream), "layer_linear_bf16")


def mfma_microbench(data_kind: int, trips: int, scratch_ptr: int, scratch_bytes: int, stream: int = 0):
    """(TFLOP/s, shader clock in GHz) of an MFMA-only loop on every CU."""
    t, c = C.c_double(0.0), C.c_double(0.0)
    _check(lib.ca_mfma_microbench(data_kind, trips, scratch_ptr, scratch_bytes, stream, C.byref(t), C.byref(c)),
           "ca_mfma_microbench")
    return t.value, c.value


class Scheduler:
    """Thin owner of a ca_sched* (Algorithm 1 control flow)."""

    def __init__(self, n_blocks: int, n_parallel: int, timesteps: Sequence[int], lag: Optional[int] = None):
        """lag None: Alg. 1 with n_parallel blocks; otherwise the lagged walk (n_parallel ignored)."""
        ts = (C.c_int32 * len(timesteps))(*timesteps)
        h = C.c_void_p()
        if lag is None:
            _check(lib.ca_sched_create(n_blocks, n_parallel, ts, len(timesteps), C.byref(h)), "ca_sched_create")
        else:
            _check(lib.ca_sched_create_lagged(n_blocks, ts, len(timesteps), lag, C.byref(h)), "ca_sched_create_lagged")
        self._h = h

    def close(self) -> None:
        if self._h:
            lib.ca_sched_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def batch(self) -> List[Tuple[int, int, int]]:
        """[(block_id, timestep_index, timestep)] of the current iteration; [] when done."""
        buf = (ca_sched_entry * 16)()
        n = C.c_int32(0)
        _check(lib.ca_sched_batch(self._h, buf, 16, C.byref(n)), "ca_sched_batch")
        return [(b.block_id, b.timestep_index, b.timestep) for b in buf[:n.value]]

    def advance(self) -> Tuple[int, int]:
        """(emitted block or -1, completed block or -1)."""
        e, c = C.c_int64(-1), C.c_int64(-1)
        _check(lib.ca_sched_advance(self._h, C.byref(e), C.byref(c)), "ca_sched_advance")
        return e.value, c.value

    def state(self) -> Tuple[int, int, int, int]:
        b, it = C.c_int64(), C.c_int64()
        tau, d = C.c_int32(), C.c_int32()
        _check(lib.ca_sched_state(self._h, C.byref(b), C.byref(tau), C.byref(d), C.byref(it)), "ca_sched_state")
        return b.value, tau.value, d.value, it.value
