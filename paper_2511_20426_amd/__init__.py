"""Block-cascaded self-attention for MI355X (gfx950): hand-written HIP kernels behind a C ABI.

`binding` mirrors include/cascade_attn.h one to one; `runner.CascadePool` adds the torch
plumbing (pool allocation, current stream) around it.  Nothing here computes: if
libcascade_attn.so is not built, importing `binding` raises.
"""
from . import binding  # noqa: F401
from .binding import (CA_BF16, CA_BIDIRECTIONAL, CA_BLOCK_CAUSAL, CA_CLEAN, CA_F32, CA_FREE,  # noqa: F401
                      CA_NOISY, CA_SINK, CascadeAttnError, Context, make_config, pool_bytes)
