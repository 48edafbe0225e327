// Internal declarations shared by the host metadata, the C-ABI layer and the kernel launchers.
// Not part of the public boundary (that is include/cascade_attn.h).
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "cascade_attn.h"

namespace ca {

constexpr int kMaxPairs = 64;      // head_dim <= 128
constexpr int kMaxKvBlocks = 32;   // sink + window + max_inflight
constexpr int kMaxInflight = 8;
// Scratch behind the bf16 pool pages: partial results of the attention kernel's split work items
// (at most kMaxPartials of them, one 256-row tile of fp32 accumulators + reference + row sum each).
constexpr int kMaxPartials = 256;
constexpr size_t kAttnScratchBytes = size_t(kMaxPartials) * 256 * 132 * 4;

// ----------------------------------------------------------------------------- host metadata
// Slot map, tags and the visibility rule; plain C++, no HIP (Sec. 3.3: shared KV pool with a
// rolling window and a sink block; Alg. 1: blocks move NOISY -> CLEAN when they complete tc).
class CacheMeta {
 public:
  static int32_t validate(const ca_config& c);
  explicit CacheMeta(const ca_config& c);

  const ca_config& cfg() const { return cfg_; }
  int block_tokens() const { return L_; }
  int pages_per_block() const { return P_; }
  int n_slots() const { return n_slots_; }
  size_t elem_bytes() const { return cfg_.dtype == CA_BF16 ? 2 : 4; }
  size_t page_elems() const { return size_t(cfg_.page_tokens) * cfg_.head_dim; }
  size_t pair_bytes() const { return 2 * page_elems() * elem_bytes(); }
  size_t page_bytes_total() const { return size_t(n_slots_) * P_ * cfg_.heads * pair_bytes(); }
  size_t pool_bytes() const { return page_bytes_total() + (cfg_.dtype == CA_BF16 ? kAttnScratchBytes : 0); }

  int32_t slot_of(int64_t g, int32_t* slot) const;       // the fixed rule, resident or not
  int32_t find(int64_t g, int32_t* slot) const;          // CA_ENOENT unless resident
  int32_t check_append(int64_t g, int32_t* slot) const;  // what append would do, no change
  void commit_append(int32_t slot, int64_t g, int32_t timestep, int32_t epoch);
  int32_t promote(int64_t g);
  int32_t evict(int64_t g);
  void retag(int32_t epoch);
  int32_t snapshot(ca_slot_info* out, int32_t cap, int32_t* n_out) const;

  // KV sequence of one forward and the block-pair mask.  kv_ids/kv_slots get n_kv entries,
  // n_vis[i] = number of leading KV entries query block i sees (the sequence is ordered so
  // that the visible set of every query block is a prefix).
  int32_t plan_forward(const int64_t* inflight, int32_t n_inflight, int32_t mode,
                       std::vector<int64_t>* kv_ids, std::vector<int32_t>* kv_slots,
                       std::vector<int32_t>* n_vis) const;

  const double* rope_freq() const { return freq_; }      // per pair, kMaxPairs entries

 private:
  ca_config cfg_;
  int L_, P_, n_slots_;
  std::vector<int64_t> block_;
  std::vector<int32_t> state_, timestep_, epoch_;
  double freq_[kMaxPairs];
};

// ----------------------------------------------------------------------------- kernel launchers
struct RopeGeom {
  double freq[kMaxPairs];   // angle per unit position for pair j
  int32_t pairs_t, pairs_h; // pairs [0,pairs_t) use the frame, [pairs_t,pairs_t+pairs_h) the row, rest the col
  int32_t grid_h, grid_w;
  int32_t heads, head_dim;
};

// y = rope(x) on [n_tokens, heads, head_dim]; token n sits at frame first_frame + n/(gh*gw).
int32_t launch_rope_apply(const RopeGeom& g, int dtype, const void* x, void* y, int64_t n_tokens,
                          int64_t first_frame, int64_t tok_stride, int64_t head_stride,
                          int64_t y_tok_stride, int64_t y_head_stride, void* stream);

// Fused K-rotation + K/V page store of n_blocks (1..kMaxInflight) blocks into their slots, one
// launch for all of them (bf16).
int32_t launch_cache_write(const RopeGeom& g, int dtype, int32_t n_blocks, const void* const* k,
                           const void* const* v, int64_t tok_stride, int64_t head_stride,
                           const int64_t* first_frame, int32_t block_tokens, int32_t page_tokens,
                           int32_t pages_per_block, const int32_t* slot, void* pool, void* stream);

struct AttnPlan {
  int32_t heads, head_dim, page_tokens, pages_per_block, block_tokens;
  int32_t n_q_blocks;                 // query blocks of this launch; query rows are n_q_blocks * block_tokens
  int32_t n_kv;                       // length of the KV sequence
  int32_t kv_slot[kMaxKvBlocks];
  int32_t n_vis[kMaxInflight];        // visible prefix length per query block
  int32_t uniform;                    // every query block sees the same prefix, n_vis[0]
};

int32_t launch_attn_f32(const AttnPlan& p, const void* q, void* out, const void* pool, void* stream);
// scratch: room for max_partials partial results (kAttnScratchBytes / kMaxPartials bytes each) of
// split work items, or nullptr / 0: then no KV walk is split.
int32_t launch_attn_bf16(const AttnPlan& p, int variant, const void* q, void* out, const void* pool,
                         void* scratch, int max_partials, void* stream);
int32_t attn_bf16_variant_ok(int variant);
// The same launch on queries that are not rotated yet: the kernel rotates them as it loads them.
// q is [rows, heads, head_dim] with the given strides; first_frame[i] is the first latent frame of
// query block i of the launch.
struct QRopePlan {
  RopeGeom geom;
  int64_t first_frame[kMaxInflight];
  int64_t tok_stride, head_stride;
};
int32_t launch_attn_bf16_rope(const AttnPlan& p, const QRopePlan& rp, int variant, const void* q, void* out,
                              const void* pool, void* scratch, int max_partials, void* stream);
// The same launch with the partial results in the library's own static device array (one copy per
// GPU, kept for the life of the process) instead of caller memory; CA_ETOOBIG if the split the
// device asks for needs more partial tiles than that array holds.  attn_static_scratch_prepare
// looks the array's address up for the current device ahead of the first launch (errors ignored:
// the launch looks again).
int32_t launch_attn_bf16_static(const AttnPlan& p, int variant, const void* q, void* out, const void* pool,
                                void* stream);
void attn_static_scratch_prepare();

int32_t run_mfma_microbench(int data_kind, int trips, void* scratch, size_t scratch_bytes, void* stream,
                            double* tflops, double* clock_ghz);
int32_t launch_gemm_bf16(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
                         int64_t ldx, int64_t ldw, int64_t ldy, void* stream);
// The QKV projection of n_blocks blocks (x rows: block b at b * block_tokens; w rows: q|k|v, head,
// dim) with the publication of K/V to the blocks' slots fused into its epilogue; q_out gets the
// packed, unrotated queries [n_blocks * block_tokens][heads * 128].
int32_t launch_gemm_qkv_publish(const RopeGeom& g, int32_t n_blocks, int32_t block_tokens, int32_t pages_per_block,
                                const int32_t* slot, const int64_t* first_frame, const void* x, int64_t ldx,
                                const void* w, int64_t ldw, int32_t K, void* q_out, void* pool, void* stream);
// Per-device facts and one-time kernel attributes, cached for up to kMaxDevices devices (thread
// safe: the cached values are idempotent and written with relaxed atomics).
constexpr int kMaxDevices = 64;
int32_t device_cu_count(int* n_cu);                                   // of the current device
int32_t ensure_dynamic_lds(const void* kernel, int bytes, int slot);  // slot: 0 attention, 1 GEMM, 2 attention rotating Q, 3 publishing GEMM
int32_t finish_launch(const char* what);   // launchers end with this: CA_OK, or CA_EDEVICE after recording HIP's last error
int32_t device_failure(const char* what, int hip_error);   // records the text, clears HIP's last error, returns CA_EDEVICE
const char* last_device_error();

}  // namespace ca

struct ca_ctx {
  ca::CacheMeta meta;
  void* pool;
  size_t pool_bytes;
  int32_t variant;
  explicit ca_ctx(const ca_config& c) : meta(c), pool(nullptr), pool_bytes(0), variant(0) {}
};
