// Host-side metadata of the shared KV pool: slot rule, block states and tags, the KV sequence
// and block-pair visibility of one forward.  Integers only, no HIP.
//
// Paper passages: a global KV pool shared by all in-flight blocks plus a fixed rolling window
// of finished blocks (Sec. 3.3); the first block optionally kept for ever as a sink (Sec. 3.3);
// blocks are promoted to clean when they complete the cache step tc (Alg. 1); a prompt switch
// re-tags but never recomputes cached K/V (Sec. 3.5); visibility is bidirectional across the
// cascade (Sec. 3.4) or block-causal (Sec. 3.2, Sec. 4.2).
#include <algorithm>
#include <cmath>

#include "ca_internal.hpp"

namespace ca {

int32_t CacheMeta::validate(const ca_config& c) {
  if (c.heads < 1 || c.head_dim < 2 || c.head_dim > 2 * kMaxPairs || (c.head_dim & 1)) return CA_EINVAL;
  if (c.frames_per_block < 1 || c.grid_h < 1 || c.grid_w < 1) return CA_EINVAL;
  if (int64_t(c.frames_per_block) * c.grid_h * c.grid_w > (1 << 24)) return CA_EINVAL;
  if (c.rope_dim_t < 0 || c.rope_dim_h < 0 || c.rope_dim_w < 0) return CA_EINVAL;
  if ((c.rope_dim_t | c.rope_dim_h | c.rope_dim_w) & 1) return CA_EINVAL;
  if (c.rope_dim_t + c.rope_dim_h + c.rope_dim_w != c.head_dim) return CA_EINVAL;
  if (!(c.rope_theta > 0.0) || !std::isfinite(c.rope_theta)) return CA_EINVAL;
  if (c.sink_blocks < 0 || c.window_blocks < 0 || c.max_inflight < 1) return CA_EINVAL;
  if (c.max_inflight > kMaxInflight) return CA_EINVAL;
  if (c.sink_blocks + c.window_blocks + c.max_inflight > kMaxKvBlocks) return CA_EINVAL;
  if (c.page_tokens < 1 || c.page_tokens > 4096) return CA_EINVAL;
  if (c.dtype != CA_F32 && c.dtype != CA_BF16) return CA_EINVAL;
  if (c.dtype == CA_BF16 && (c.head_dim != 128 || c.page_tokens != 128)) return CA_EUNSUPPORTED;
  if (c.dtype == CA_F32 && c.head_dim != 32 && c.head_dim != 64 && c.head_dim != 128) return CA_EUNSUPPORTED;
  return CA_OK;
}

CacheMeta::CacheMeta(const ca_config& c) : cfg_(c) {
  L_ = c.frames_per_block * c.grid_h * c.grid_w;
  P_ = (L_ + c.page_tokens - 1) / c.page_tokens;
  n_slots_ = c.sink_blocks + c.window_blocks + c.max_inflight;
  block_.assign(n_slots_, -1);
  state_.assign(n_slots_, CA_FREE);
  timestep_.assign(n_slots_, 0);
  epoch_.assign(n_slots_, 0);
  std::fill(freq_, freq_ + kMaxPairs, 0.0);
  const int dims[3] = {c.rope_dim_t, c.rope_dim_h, c.rope_dim_w};
  int pair = 0;
  for (int a = 0; a < 3; ++a)
    for (int j = 0; j < dims[a] / 2; ++j)
      freq_[pair++] = std::pow(c.rope_theta, -2.0 * double(j) / double(dims[a]));
}

int32_t CacheMeta::slot_of(int64_t g, int32_t* slot) const {
  if (g < 0) return CA_EINVAL;
  const int64_t S = cfg_.sink_blocks;
  const int64_t ring = cfg_.window_blocks + cfg_.max_inflight;
  *slot = g < S ? int32_t(g) : int32_t(S + (g - S) % ring);
  return CA_OK;
}

int32_t CacheMeta::find(int64_t g, int32_t* slot) const {
  int32_t s;
  if (int32_t rc = slot_of(g, &s)) return rc;
  if (state_[s] == CA_FREE || block_[s] != g) return CA_ENOENT;
  *slot = s;
  return CA_OK;
}

int32_t CacheMeta::check_append(int64_t g, int32_t* slot) const {
  int32_t s;
  if (int32_t rc = slot_of(g, &s)) return rc;
  if (state_[s] != CA_FREE && block_[s] != g) return CA_ENOSPC;
  if (state_[s] == CA_CLEAN || state_[s] == CA_SINK) return CA_ESTATE;
  *slot = s;
  return CA_OK;
}

void CacheMeta::commit_append(int32_t slot, int64_t g, int32_t timestep, int32_t epoch) {
  block_[slot] = g;
  state_[slot] = CA_NOISY;
  timestep_[slot] = timestep;
  epoch_[slot] = epoch;
}

int32_t CacheMeta::promote(int64_t g) {
  int32_t s;
  if (int32_t rc = find(g, &s)) return rc;
  if (state_[s] != CA_NOISY) return CA_ESTATE;
  state_[s] = g < cfg_.sink_blocks ? CA_SINK : CA_CLEAN;
  return CA_OK;
}

int32_t CacheMeta::evict(int64_t g) {
  int32_t s;
  if (int32_t rc = find(g, &s)) return rc;
  if (state_[s] == CA_SINK) return CA_ESTATE;
  block_[s] = -1;
  state_[s] = CA_FREE;
  timestep_[s] = 0;
  epoch_[s] = 0;
  return CA_OK;
}

void CacheMeta::retag(int32_t epoch) {
  for (int s = 0; s < n_slots_; ++s)
    if (state_[s] == CA_NOISY) epoch_[s] = epoch;
}

int32_t CacheMeta::snapshot(ca_slot_info* out, int32_t cap, int32_t* n_out) const {
  if (!n_out || cap < 0 || (cap > 0 && !out)) return CA_EINVAL;
  int32_t n = 0;
  for (int s = 0; s < n_slots_; ++s) {
    if (state_[s] == CA_FREE) continue;
    if (n < cap) {
      out[n].slot = s;
      out[n].state = state_[s];
      out[n].block_id = block_[s];
      out[n].timestep = timestep_[s];
      out[n].prompt_epoch = epoch_[s];
    }
    ++n;
  }
  *n_out = n;
  return CA_OK;
}

int32_t CacheMeta::plan_forward(const int64_t* inflight, int32_t n_inflight, int32_t mode,
                                std::vector<int64_t>* kv_ids, std::vector<int32_t>* kv_slots,
                                std::vector<int32_t>* n_vis) const {
  if (!inflight || n_inflight < 1 || n_inflight > cfg_.max_inflight) return CA_EINVAL;
  if (mode != CA_BIDIRECTIONAL && mode != CA_BLOCK_CAUSAL) return CA_EINVAL;
  for (int i = 0; i < n_inflight; ++i) {
    if (i > 0 && inflight[i] <= inflight[i - 1]) return CA_EINVAL;
    int32_t s;
    if (int32_t rc = find(inflight[i], &s)) return rc;
    if (state_[s] != CA_NOISY) return CA_ESTATE;
  }
  kv_ids->clear();
  kv_slots->clear();
  n_vis->clear();
  // finished blocks first: sinks, then the clean window, each by ascending block index
  for (int pass = 0; pass < 2; ++pass) {
    const int want = pass == 0 ? CA_SINK : CA_CLEAN;
    std::vector<std::pair<int64_t, int32_t>> v;
    for (int s = 0; s < n_slots_; ++s)
      if (state_[s] == want) v.emplace_back(block_[s], s);
    std::sort(v.begin(), v.end());
    for (auto& e : v) {
      kv_ids->push_back(e.first);
      kv_slots->push_back(e.second);
    }
  }
  const int32_t n_cache = int32_t(kv_ids->size());
  for (int i = 0; i < n_inflight; ++i) {
    int32_t s;
    find(inflight[i], &s);
    kv_ids->push_back(inflight[i]);
    kv_slots->push_back(s);
    n_vis->push_back(mode == CA_BIDIRECTIONAL ? n_cache + n_inflight : n_cache + i + 1);
  }
  return CA_OK;
}

}  // namespace ca
