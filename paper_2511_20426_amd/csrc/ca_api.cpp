// C-ABI entry points (include/cascade_attn.h): argument checks, metadata update, kernel launch.
// Every failing call returns before touching metadata or the GPU.
#include <cmath>
#include <new>

#include "ca_internal.hpp"
#include "cascade_attn_lab.h"

namespace {

ca::RopeGeom rope_geom(const ca::CacheMeta& m) {
  ca::RopeGeom g{};
  const ca_config& c = m.cfg();
  for (int i = 0; i < ca::kMaxPairs; ++i) g.freq[i] = m.rope_freq()[i];
  g.pairs_t = c.rope_dim_t / 2;
  g.pairs_h = c.rope_dim_h / 2;
  g.grid_h = c.grid_h;
  g.grid_w = c.grid_w;
  g.heads = c.heads;
  g.head_dim = c.head_dim;
  return g;
}

// A [token, head, dim] view must address whole 8-element groups on 16-byte (bf16) or
// 32-byte (fp32) boundaries: the kernels move 8 elements at a time.
bool strides_ok(const ca_config& c, const void* p, int64_t tok_stride, int64_t head_stride) {
  if (tok_stride < 0 || head_stride < 0) return false;
  if (head_stride < c.head_dim && c.heads > 1) return false;
  if (tok_stride < c.head_dim) return false;
  if ((tok_stride % 8) || (head_stride % 8)) return false;
  if (reinterpret_cast<uintptr_t>(p) % 16) return false;
  return true;
}

}  // namespace

extern "C" {

size_t ca_pool_bytes(const ca_config* cfg) {
  if (!cfg || ca::CacheMeta::validate(*cfg) != CA_OK) return 0;
  return ca::CacheMeta(*cfg).pool_bytes();
}

int32_t ca_create(const ca_config* cfg, void* pool_dev, size_t pool_bytes, ca_ctx** out) {
  if (!cfg || !out) return CA_EINVAL;
  if (int32_t rc = ca::CacheMeta::validate(*cfg)) return rc;
  if ((pool_dev == nullptr) != (pool_bytes == 0)) return CA_EINVAL;
  ca_ctx* ctx = new (std::nothrow) ca_ctx(*cfg);
  if (!ctx) return CA_EINVAL;
  if (pool_dev) {
    if (pool_bytes < ctx->meta.pool_bytes() || (reinterpret_cast<uintptr_t>(pool_dev) & 255)) {
      delete ctx;
      return CA_EINVAL;
    }
  }
  ctx->pool = pool_dev;
  ctx->pool_bytes = pool_bytes;
  if (pool_dev && cfg->dtype == CA_BF16) ca::attn_static_scratch_prepare();   // for cascade_attn_forward_static
  *out = ctx;
  return CA_OK;
}

int32_t ca_destroy(ca_ctx* ctx) {
  if (!ctx) return CA_EINVAL;
  delete ctx;
  return CA_OK;
}

int32_t kv_cache_append(ca_ctx* ctx, int64_t block_id, int32_t timestep, int32_t prompt_epoch,
                        const void* k_dev, const void* v_dev, int64_t tok_stride,
                        int64_t head_stride, void* hip_stream, int32_t* slot_out) {
  return kv_cache_append_batch(ctx, 1, &block_id, &timestep, prompt_epoch, &k_dev, &v_dev, tok_stride,
                               head_stride, hip_stream, slot_out);
}

int32_t kv_cache_append_batch(ca_ctx* ctx, int32_t n_blocks, const int64_t* block_ids,
                              const int32_t* timesteps, int32_t prompt_epoch, const void* const* k_dev,
                              const void* const* v_dev, int64_t tok_stride, int64_t head_stride,
                              void* hip_stream, int32_t* slots_out) {
  if (!ctx || !block_ids || !timesteps || n_blocks < 1 || n_blocks > ca::kMaxInflight) return CA_EINVAL;
  // the entries are applied in order to a copy of the metadata: entry i sees what entries
  // 0..i-1 did, and nothing has changed if any of them fails
  ca::CacheMeta next = ctx->meta;
  int32_t slots[ca::kMaxInflight];
  int64_t first_frame[ca::kMaxInflight];
  for (int i = 0; i < n_blocks; ++i) {
    if (int32_t rc = next.check_append(block_ids[i], &slots[i])) return rc;
    for (int j = 0; j < i; ++j)
      if (block_ids[j] == block_ids[i]) return CA_EINVAL;      // one launch writes a slot once
    next.commit_append(slots[i], block_ids[i], timesteps[i], prompt_epoch);
    first_frame[i] = int64_t(next.cfg().frames_per_block) * block_ids[i];
  }
  if (ctx->pool) {
    if (!k_dev || !v_dev) return CA_EINVAL;
    const ca_config& c = next.cfg();
    for (int i = 0; i < n_blocks; ++i) {
      if (!k_dev[i] || !v_dev[i]) return CA_EINVAL;
      if (!strides_ok(c, k_dev[i], tok_stride, head_stride) || !strides_ok(c, v_dev[i], tok_stride, head_stride))
        return CA_EINVAL;
    }
    const int32_t rc = ca::launch_cache_write(rope_geom(next), c.dtype, n_blocks, k_dev, v_dev, tok_stride,
                                              head_stride, first_frame, next.block_tokens(), c.page_tokens,
                                              next.pages_per_block(), slots, ctx->pool, hip_stream);
    if (rc != CA_OK) return rc;
  }
  ctx->meta = next;
  if (slots_out)
    for (int i = 0; i < n_blocks; ++i) slots_out[i] = slots[i];
  return CA_OK;
}

int32_t layer_qkv_publish(ca_ctx* ctx, int32_t n_blocks, const int64_t* block_ids, const int32_t* timesteps,
                          int32_t prompt_epoch, const void* x_dev, int64_t ldx, const void* w_qkv_dev, int64_t ldw,
                          int32_t k_in, void* q_out_dev, void* hip_stream, int32_t* slots_out) {
  if (!ctx || !block_ids || !timesteps || n_blocks < 1 || n_blocks > ca::kMaxInflight) return CA_EINVAL;
  if (!ctx->pool) return CA_ENOPOOL;
  if (ctx->meta.cfg().dtype != CA_BF16) return CA_EUNSUPPORTED;
  if (!x_dev || !w_qkv_dev || !q_out_dev) return CA_EINVAL;
  if ((reinterpret_cast<uintptr_t>(x_dev) | reinterpret_cast<uintptr_t>(w_qkv_dev) |
       reinterpret_cast<uintptr_t>(q_out_dev)) & 15)
    return CA_EINVAL;
  // as kv_cache_append_batch: the entries take effect in order on a copy, all or none
  ca::CacheMeta next = ctx->meta;
  int32_t slots[ca::kMaxInflight];
  int64_t first_frame[ca::kMaxInflight];
  for (int i = 0; i < n_blocks; ++i) {
    if (int32_t rc = next.check_append(block_ids[i], &slots[i])) return rc;
    for (int j = 0; j < i; ++j)
      if (block_ids[j] == block_ids[i]) return CA_EINVAL;
    next.commit_append(slots[i], block_ids[i], timesteps[i], prompt_epoch);
    first_frame[i] = int64_t(next.cfg().frames_per_block) * block_ids[i];
  }
  const int32_t rc = ca::launch_gemm_qkv_publish(rope_geom(next), n_blocks, next.block_tokens(), next.pages_per_block(),
                                                 slots, first_frame, x_dev, ldx, w_qkv_dev, ldw, k_in, q_out_dev,
                                                 ctx->pool, hip_stream);
  if (rc != CA_OK) return rc;
  ctx->meta = next;
  if (slots_out)
    for (int i = 0; i < n_blocks; ++i) slots_out[i] = slots[i];
  return CA_OK;
}

int32_t kv_cache_promote(ca_ctx* ctx, int64_t block_id) {
  return ctx ? ctx->meta.promote(block_id) : CA_EINVAL;
}

int32_t kv_cache_evict(ca_ctx* ctx, int64_t block_id) {
  return ctx ? ctx->meta.evict(block_id) : CA_EINVAL;
}

int32_t kv_cache_retag(ca_ctx* ctx, int32_t new_prompt_epoch) {
  if (!ctx) return CA_EINVAL;
  ctx->meta.retag(new_prompt_epoch);
  return CA_OK;
}

int32_t kv_cache_snapshot(const ca_ctx* ctx, ca_slot_info* out, int32_t cap, int32_t* n_out) {
  return ctx ? ctx->meta.snapshot(out, cap, n_out) : CA_EINVAL;
}

int32_t kv_cache_page_index(const ca_ctx* ctx, int64_t block_id, int32_t page, int32_t head,
                            int64_t* index_out) {
  if (!ctx || !index_out) return CA_EINVAL;
  const ca::CacheMeta& m = ctx->meta;
  if (page < 0 || page >= m.pages_per_block() || head < 0 || head >= m.cfg().heads) return CA_EINVAL;
  int32_t slot;
  if (int32_t rc = m.find(block_id, &slot)) return rc;
  *index_out = (int64_t(slot) * m.pages_per_block() + page) * m.cfg().heads + head;
  return CA_OK;
}

int32_t rope3d_apply_strided(const ca_ctx* ctx, const void* x_dev, int64_t x_tok_stride, int64_t x_head_stride,
                             void* y_dev, int64_t y_tok_stride, int64_t y_head_stride, int64_t n_tokens,
                             int64_t first_frame, void* hip_stream) {
  if (!ctx || n_tokens < 0 || first_frame < 0) return CA_EINVAL;
  if (!ctx->pool) return CA_ENOPOOL;
  if (n_tokens == 0) return CA_OK;
  if (!x_dev || !y_dev) return CA_EINVAL;
  const ca::CacheMeta& m = ctx->meta;
  if (!strides_ok(m.cfg(), x_dev, x_tok_stride, x_head_stride) ||
      !strides_ok(m.cfg(), y_dev, y_tok_stride, y_head_stride))
    return CA_EINVAL;
  return ca::launch_rope_apply(rope_geom(m), m.cfg().dtype, x_dev, y_dev, n_tokens, first_frame,
                               x_tok_stride, x_head_stride, y_tok_stride, y_head_stride, hip_stream);
}

int32_t rope3d_apply(const ca_ctx* ctx, const void* x_dev, void* y_dev, int64_t n_tokens,
                     int64_t first_frame, int64_t tok_stride, int64_t head_stride,
                     void* hip_stream) {
  return rope3d_apply_strided(ctx, x_dev, tok_stride, head_stride, y_dev, tok_stride, head_stride, n_tokens,
                              first_frame, hip_stream);
}

}  // extern "C"

namespace {

// partials: where the bf16 kernel's split work items put their partial results
enum class Partials { kInPool, kStatic };

// q_strides: null for rotated, contiguous queries; else {token stride, head stride} of unrotated
// queries that the kernel rotates itself
int32_t forward_impl(ca_ctx* ctx, const void* q_dev, const int64_t* inflight_block_ids, int32_t n_inflight,
                     int32_t first, int32_t count, int32_t mode, void* out_dev, void* hip_stream, Partials where,
                     const int64_t* q_strides = nullptr) {
  if (!ctx) return CA_EINVAL;
  const ca::CacheMeta& m = ctx->meta;
  std::vector<int64_t> ids;
  std::vector<int32_t> slots, n_vis;
  if (int32_t rc = m.plan_forward(inflight_block_ids, n_inflight, mode, &ids, &slots, &n_vis)) return rc;
  if (first < 0 || count < 1 || first > n_inflight - count) return CA_EINVAL;
  if (!ctx->pool) return CA_ENOPOOL;
  if (!q_dev || !out_dev) return CA_EINVAL;
  if ((reinterpret_cast<uintptr_t>(q_dev) | reinterpret_cast<uintptr_t>(out_dev)) & 15) return CA_EINVAL;
  const ca_config& c = m.cfg();
  ca::AttnPlan p{};
  p.heads = c.heads;
  p.head_dim = c.head_dim;
  p.page_tokens = c.page_tokens;
  p.pages_per_block = m.pages_per_block();
  p.block_tokens = m.block_tokens();
  p.n_q_blocks = count;
  p.n_kv = int32_t(ids.size());
  p.uniform = 1;
  for (int i = 0; i < p.n_kv; ++i) p.kv_slot[i] = slots[i];
  for (int i = 0; i < count; ++i) {
    p.n_vis[i] = n_vis[first + i];
    if (p.n_vis[i] != p.n_vis[0]) p.uniform = 0;
  }
  if (q_strides) {
    if (c.dtype != CA_BF16) return CA_EUNSUPPORTED;
    if (!strides_ok(c, q_dev, q_strides[0], q_strides[1])) return CA_EINVAL;
    ca::QRopePlan rp{};
    rp.geom = rope_geom(m);
    for (int i = 0; i < count; ++i) rp.first_frame[i] = int64_t(c.frames_per_block) * inflight_block_ids[first + i];
    rp.tok_stride = q_strides[0];
    rp.head_stride = q_strides[1];
    return ca::launch_attn_bf16_rope(p, rp, ctx->variant, q_dev, out_dev, ctx->pool,
                                     static_cast<uint8_t*>(ctx->pool) + m.page_bytes_total(), ca::kMaxPartials,
                                     hip_stream);
  }
  if (c.dtype != CA_BF16) return ca::launch_attn_f32(p, q_dev, out_dev, ctx->pool, hip_stream);   // no scratch at all
  if (where == Partials::kStatic)
    return ca::launch_attn_bf16_static(p, ctx->variant, q_dev, out_dev, ctx->pool, hip_stream);
  return ca::launch_attn_bf16(p, ctx->variant, q_dev, out_dev, ctx->pool,
                              static_cast<uint8_t*>(ctx->pool) + m.page_bytes_total(), ca::kMaxPartials, hip_stream);
}

}  // namespace

extern "C" {

int32_t cascade_attn_forward(ca_ctx* ctx, const void* q_dev, const int64_t* inflight_block_ids,
                             int32_t n_inflight, int32_t mode, void* out_dev, void* hip_stream) {
  return forward_impl(ctx, q_dev, inflight_block_ids, n_inflight, 0, n_inflight, mode, out_dev, hip_stream,
                      Partials::kInPool);
}

int32_t cascade_attn_forward_share(ca_ctx* ctx, const void* q_dev, const int64_t* inflight_block_ids,
                                   int32_t n_inflight, int32_t first, int32_t count, int32_t mode,
                                   void* out_dev, void* hip_stream) {
  return forward_impl(ctx, q_dev, inflight_block_ids, n_inflight, first, count, mode, out_dev, hip_stream,
                      Partials::kInPool);
}

int32_t cascade_attn_forward_rope(ca_ctx* ctx, const void* q_dev, int64_t q_tok_stride, int64_t q_head_stride,
                                  const int64_t* inflight_block_ids, int32_t n_inflight, int32_t mode,
                                  void* out_dev, void* hip_stream) {
  const int64_t strides[2] = {q_tok_stride, q_head_stride};
  return forward_impl(ctx, q_dev, inflight_block_ids, n_inflight, 0, n_inflight, mode, out_dev, hip_stream,
                      Partials::kInPool, strides);
}

int32_t cascade_attn_forward_static(ca_ctx* ctx, const void* q_dev, const int64_t* inflight_block_ids,
                                    int32_t n_inflight, int32_t mode, void* out_dev, void* hip_stream) {
  return forward_impl(ctx, q_dev, inflight_block_ids, n_inflight, 0, n_inflight, mode, out_dev, hip_stream,
                      Partials::kStatic);
}

int32_t ca_debug_visibility(const ca_ctx* ctx, const int64_t* inflight_block_ids,
                            int32_t n_inflight, int32_t mode, uint8_t* vis, int64_t* kv_block_ids,
                            int32_t cap, int32_t* n_kv_out) {
  if (!ctx || !vis || !kv_block_ids || !n_kv_out) return CA_EINVAL;
  std::vector<int64_t> ids;
  std::vector<int32_t> slots, n_vis;
  if (int32_t rc = ctx->meta.plan_forward(inflight_block_ids, n_inflight, mode, &ids, &slots, &n_vis))
    return rc;
  const int32_t n_kv = int32_t(ids.size());
  if (cap < n_kv) return CA_EINVAL;
  for (int r = 0; r < n_kv; ++r) kv_block_ids[r] = ids[r];
  for (int i = 0; i < n_inflight; ++i)
    for (int r = 0; r < n_kv; ++r) vis[i * n_kv + r] = r < n_vis[i] ? 1 : 0;
  *n_kv_out = n_kv;
  return CA_OK;
}

int32_t layer_linear_bf16(const void* x_dev, const void* w_dev, void* y_dev, int64_t m_rows, int32_t n_out,
                          int32_t k_in, int64_t ldx, int64_t ldw, int64_t ldy, void* hip_stream) {
  if (!x_dev || !w_dev || !y_dev) return CA_EINVAL;
  if ((reinterpret_cast<uintptr_t>(x_dev) | reinterpret_cast<uintptr_t>(w_dev) | reinterpret_cast<uintptr_t>(y_dev)) & 15)
    return CA_EINVAL;
  return ca::launch_gemm_bf16(x_dev, w_dev, y_dev, m_rows, n_out, k_in, ldx, ldw, ldy, hip_stream);
}

int32_t ca_mfma_microbench(int32_t data_kind, int32_t trips, void* scratch_dev, size_t scratch_bytes,
                           void* hip_stream, double* tflops, double* clock_ghz) {
  if ((data_kind != 0 && data_kind != 1) || trips < 1 || trips > (1 << 24) || !scratch_dev) return CA_EINVAL;
  return ca::run_mfma_microbench(data_kind, trips, scratch_dev, scratch_bytes, hip_stream, tflops, clock_ghz);
}

int32_t ca_set_kernel_variant(ca_ctx* ctx, int32_t variant) {
  if (!ctx) return CA_EINVAL;
  if (int32_t rc = ca::attn_bf16_variant_ok(variant)) return rc;
  ctx->variant = variant;
  return CA_OK;
}

const char* ca_strerror(int32_t code) {
  switch (code) {
    case CA_OK: return "ok";
    case CA_EINVAL: return "invalid argument";
    case CA_ENOSPC: return "slot still held by another block";
    case CA_ENOENT: return "block not resident";
    case CA_ESTATE: return "block is in the wrong state for this call";
    case CA_EUNSUPPORTED: return "dtype / head_dim / page size not supported";
    case CA_ENOPOOL: return "context has no device pool";
    case CA_EDEVICE: return "HIP launch failed";
    case CA_ETOOBIG: return "the forward needs more partial-result tiles than the static scratch area holds";
    default: return "unknown error";
  }
}

const char* ca_last_device_error(void) { return ca::last_device_error(); }

}  // extern "C"
