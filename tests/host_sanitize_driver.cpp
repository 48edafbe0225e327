// Host-only exercise of the C-ABI layer, the cache metadata and the scheduler, built by
// tests/test_host_sanitizers.py with -fsanitize=address,undefined (no HIP: the kernel
// launchers are replaced by the stubs below, which only check what they are handed).
// Exit code 0 = every call behaved; the sanitizers abort on anything else.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ca_internal.hpp"
#include "cascade_attn_lab.h"

namespace ca {

static int g_launches = 0;

int32_t launch_rope_apply(const RopeGeom&, int, const void* x, void* y, int64_t n, int64_t, int64_t, int64_t,
                          int64_t, int64_t, void*) {
  ++g_launches;
  return x && y && n > 0 ? CA_OK : CA_EDEVICE;
}
int32_t launch_cache_write(const RopeGeom& g, int, int32_t n_blocks, const void* const* k, const void* const* v,
                           int64_t, int64_t, const int64_t* first_frame, int32_t, int32_t, int32_t,
                           const int32_t* slot, void* pool, void*) {
  ++g_launches;
  if (!pool || n_blocks < 1 || n_blocks > kMaxInflight || g.heads < 1) return CA_EDEVICE;
  for (int i = 0; i < n_blocks; ++i)
    if (!k[i] || !v[i] || first_frame[i] < 0 || slot[i] < 0) return CA_EDEVICE;
  return CA_OK;
}
int32_t launch_attn_f32(const AttnPlan& p, const void* q, void* out, const void* pool, void*) {
  ++g_launches;
  for (int i = 0; i < p.n_q_blocks; ++i)
    if (p.n_vis[i] < 1 || p.n_vis[i] > p.n_kv) return CA_EDEVICE;
  return q && out && pool ? CA_OK : CA_EDEVICE;
}
int32_t launch_attn_bf16(const AttnPlan& p, int, const void* q, void* out, const void* pool, void* scratch,
                         int max_partials, void*) {
  ++g_launches;
  for (int i = 0; i < p.n_q_blocks; ++i)
    if (p.n_vis[i] < 1 || p.n_vis[i] > p.n_kv) return CA_EDEVICE;
  for (int i = 0; i < p.n_kv; ++i)
    if (p.kv_slot[i] < 0) return CA_EDEVICE;
  return q && out && pool && scratch && max_partials > 0 ? CA_OK : CA_EDEVICE;
}
int32_t launch_attn_bf16_rope(const AttnPlan& p, const QRopePlan& rp, int, const void* q, void* out, const void* pool,
                              void* scratch, int, void*) {
  ++g_launches;
  for (int i = 0; i < p.n_q_blocks; ++i)
    if (rp.first_frame[i] < 0) return CA_EDEVICE;
  return q && out && pool && scratch && rp.tok_stride >= rp.geom.head_dim ? CA_OK : CA_EDEVICE;
}
int32_t launch_attn_bf16_static(const AttnPlan& p, int, const void* q, void* out, const void* pool, void*) {
  ++g_launches;
  return q && out && pool && p.n_q_blocks > 0 ? CA_OK : CA_EDEVICE;
}
void attn_static_scratch_prepare() {}
int32_t attn_bf16_variant_ok(int variant) { return variant == 0 || variant == 1 ? CA_OK : CA_EINVAL; }
int32_t run_mfma_microbench(int, int, void*, size_t, void*, double*, double*) { return CA_OK; }
int32_t launch_gemm_bf16(const void*, const void*, void*, int64_t, int32_t n, int32_t k, int64_t, int64_t, int64_t,
                         void*) {
  return (n % 8 || k % 128) ? CA_EUNSUPPORTED : CA_OK;
}
int32_t launch_gemm_qkv_publish(const RopeGeom& g, int32_t n_blocks, int32_t block_tokens, int32_t pages, const int32_t* slot,
                                const int64_t* first_frame, const void* x, int64_t ldx, const void* w, int64_t, int32_t k,
                                void* q_out, void* pool, void*) {
  ++g_launches;
  if (g.heads % 2 || k % 128) return CA_EUNSUPPORTED;
  for (int i = 0; i < n_blocks; ++i)
    if (slot[i] < 0 || first_frame[i] < 0) return CA_EDEVICE;
  return x && w && q_out && pool && ldx >= k && block_tokens > 0 && pages > 0 ? CA_OK : CA_EDEVICE;
}
const char* last_device_error() { return ""; }

}  // namespace ca

#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      std::exit(1);                                                          \
    }                                                                        \
  } while (0)

static ca_config config(int dtype, int sink, int window, int inflight) {
  ca_config c{};
  c.heads = 3; c.head_dim = 128;
  c.frames_per_block = 3; c.grid_h = 7; c.grid_w = 11;
  c.rope_dim_t = 44; c.rope_dim_h = 42; c.rope_dim_w = 42;
  c.rope_theta = 10000.0;
  c.sink_blocks = sink; c.window_blocks = window; c.max_inflight = inflight;
  c.page_tokens = 128; c.dtype = dtype;
  return c;
}

// A rollout of Alg. 1 driven by the scheduler over a context with a (fake) pool: appends in one
// launch per iteration, a forward and a share of it, promote / evict, a prompt switch, snapshots
// into buffers that are too small, and every error path in between.
static void rollout(int dtype, int sink, int window, int lag) {
  const ca_config cfg = config(dtype, sink, window, 5);
  const size_t bytes = ca_pool_bytes(&cfg);
  CHECK(bytes > 0);
  std::vector<unsigned char> fake_pool(512, 0);          // never dereferenced by the stubs
  void* pool = reinterpret_cast<void*>((reinterpret_cast<uintptr_t>(fake_pool.data()) + 255) & ~uintptr_t(255));
  ca_ctx* ctx = nullptr;
  CHECK(ca_create(&cfg, pool, bytes - 1, &ctx) == CA_EINVAL);
  CHECK(ca_create(&cfg, pool, bytes, &ctx) == CA_OK);
  const int32_t T[5] = {1000, 750, 500, 250, 0};
  ca_sched* sched = nullptr;
  const int64_t n_blocks = 23;
  CHECK(ca_sched_create_lagged(n_blocks, T, 5, lag, &sched) == CA_OK);
  alignas(16) static unsigned short tensor[8];           // stands for K, V, Q, O: only its address is used
  std::vector<int64_t> clean;
  int iterations = 0;
  for (;;) {
    ca_sched_entry batch[8];
    int32_t n = 0;
    CHECK(ca_sched_batch(sched, batch, 0, &n) == (iterations < lag * (n_blocks - 1) + 5 ? CA_EINVAL : CA_OK));
    CHECK(ca_sched_batch(sched, batch, 8, &n) == CA_OK);
    if (n == 0) break;
    int64_t ids[8];
    int32_t ts[8], slots[8];
    const void* kv[8];
    for (int i = 0; i < n; ++i) {
      ids[i] = batch[i].block_id;
      ts[i] = batch[i].timestep;
      kv[i] = tensor;
    }
    CHECK(kv_cache_append_batch(ctx, n, ids, ts, iterations / 9, kv, kv, 3 * 128, 128, nullptr, slots) == CA_OK);
    CHECK(kv_cache_append_batch(ctx, n, ids, ts, 0, kv, kv, 3 * 128 + 1, 128, nullptr, slots) == CA_EINVAL);
    for (int mode = 0; mode < 2; ++mode) {
      CHECK(cascade_attn_forward(ctx, tensor, ids, n, mode, tensor, nullptr) == CA_OK);
      CHECK(cascade_attn_forward_share(ctx, tensor, ids, n, n - 1, 1, mode, tensor, nullptr) == CA_OK);
      CHECK(cascade_attn_forward_static(ctx, tensor, ids, n, mode, tensor, nullptr) == CA_OK);
      CHECK(cascade_attn_forward_rope(ctx, tensor, 3 * 128 * cfg.heads, 128, ids, n, mode, tensor, nullptr) ==
            (dtype == CA_BF16 ? CA_OK : CA_EUNSUPPORTED));
      CHECK(cascade_attn_forward_rope(ctx, tensor, 64, 128, ids, n, mode, tensor, nullptr) ==
            (dtype == CA_BF16 ? CA_EINVAL : CA_EUNSUPPORTED));
      CHECK(cascade_attn_forward_static(ctx, nullptr, ids, n, mode, tensor, nullptr) == CA_EINVAL);
      CHECK(cascade_attn_forward_share(ctx, tensor, ids, n, n, 1, mode, tensor, nullptr) == CA_EINVAL);
      uint8_t vis[8 * 32];
      int64_t kv_ids[32];
      int32_t n_kv = 0;
      CHECK(ca_debug_visibility(ctx, ids, n, mode, vis, kv_ids, 32, &n_kv) == CA_OK);
      CHECK(n_kv >= n && n_kv <= sink + window + 5);
      CHECK(ca_debug_visibility(ctx, ids, n, mode, vis, kv_ids, n_kv - 1, &n_kv) == CA_EINVAL);
    }
    CHECK(rope3d_apply(ctx, tensor, tensor, 17, 3 * ids[0], 3 * 128, 128, nullptr) == CA_OK);
    if (iterations == 11) CHECK(kv_cache_retag(ctx, 7) == CA_OK);
    int64_t emitted = -2, completed = -2;
    CHECK(ca_sched_advance(sched, &emitted, &completed) == CA_OK);
    if (completed >= 0) {
      CHECK(kv_cache_promote(ctx, completed) == CA_OK);
      CHECK(kv_cache_promote(ctx, completed) == CA_ESTATE);
      if (completed >= sink) {
        clean.push_back(completed);
        if (int(clean.size()) > window) {
          CHECK(kv_cache_evict(ctx, clean.front()) == CA_OK);
          CHECK(kv_cache_evict(ctx, clean.front()) == CA_ENOENT);
          clean.erase(clean.begin());
        }
      }
    }
    ca_slot_info info[32];
    int32_t n_slots = 0;
    CHECK(kv_cache_snapshot(ctx, info, 2, &n_slots) == CA_OK);      // fewer entries than slots in use
    CHECK(kv_cache_snapshot(ctx, nullptr, 0, &n_slots) == CA_OK);
    CHECK(n_slots <= sink + window + 5);
    CHECK(kv_cache_snapshot(ctx, info, 32, &n_slots) == CA_OK);
    for (int i = 0; i < n_slots; ++i) {
      int64_t index = -1;
      CHECK(kv_cache_page_index(ctx, info[i].block_id, 0, cfg.heads - 1, &index) == CA_OK && index >= 0);
    }
    ++iterations;
  }
  CHECK(iterations == lag * (n_blocks - 1) + 5);
  int64_t e, c;
  CHECK(ca_sched_advance(sched, &e, &c) == CA_ESTATE);
  CHECK(ca_sched_destroy(sched) == CA_OK);
  CHECK(ca_destroy(ctx) == CA_OK);
}

int main() {
  for (int dtype : {CA_BF16, CA_F32})
    for (int sink : {0, 1})
      for (int lag : {1, 2, 3, 5}) rollout(dtype, sink, dtype == CA_BF16 ? 6 : 2, lag);
  // the limits of a context, and a metadata-only one
  ca_config big = config(CA_BF16, 1, 23, 8);
  CHECK(ca_pool_bytes(&big) > 0);
  big.window_blocks = 24;
  CHECK(ca_pool_bytes(&big) == 0);
  ca_config meta_only = config(CA_BF16, 1, 6, 5);
  ca_ctx* ctx = nullptr;
  CHECK(ca_create(&meta_only, nullptr, 0, &ctx) == CA_OK);
  int32_t slot = -1;
  CHECK(kv_cache_append(ctx, 4, 500, 0, nullptr, nullptr, 0, 0, nullptr, &slot) == CA_OK && slot == 4);
  const int64_t id = 4;
  CHECK(cascade_attn_forward(ctx, nullptr, &id, 1, CA_BIDIRECTIONAL, nullptr, nullptr) == CA_ENOPOOL);
  CHECK(ca_destroy(ctx) == CA_OK);
  alignas(16) static unsigned short m[16];
  CHECK(layer_linear_bf16(m + 1, m, m, 5, 256, 128, 128, 128, 256, nullptr) == CA_EINVAL);        // misaligned x
  CHECK(layer_linear_bf16(m, m, m, 5, 256, 128, 128, 128, 256, nullptr) == CA_OK);
  CHECK(layer_linear_bf16(m, m, m, 5, 255, 128, 128, 128, 256, nullptr) == CA_EUNSUPPORTED);
  CHECK(std::strlen(ca_strerror(CA_ENOSPC)) > 0);
  CHECK(ca::g_launches > 0);
  std::puts("host sanitizer driver: ok");
  return 0;
}
