// Host-side cascade scheduler: the control flow of Algorithm 1 (the multi-GPU cascade schedule),
// integers only, generalised by the lag between consecutive blocks.
//
// Every block walks the timestep list T one entry per iteration; block j enters `lag` iterations
// after block j-1.  In iteration n the batch therefore holds the blocks j with
// 0 <= n - lag*j < |T|, block j at T[n - lag*j] (older blocks are cleaner); a block that ran at t0
// (the second-to-last entry of T) is emitted, one that ran at tc (the last entry) is complete.
// lag = 1 is Algorithm 1 as listed with G = |T| parallel blocks: state (b, tau, d) = (oldest block
// in flight, its timestep index, batch size - 1) then takes exactly the listing's values.  The
// listing itself is self-consistent only for G = |T| (otherwise a new block would enter in the
// middle of the schedule), so other degrees of cascading are expressed through the lag instead:
// lag = 5, 3, 2, 1 keep at most 1, 2, 3, 5 blocks in flight (the cascade types P1..P4 of the
// ablation, Sec. 4.2 / Fig. 7, as far as the text fixes them).
#include <new>
#include <vector>

#include "cascade_attn.h"

struct ca_sched {
  int64_t n_blocks;
  int32_t lag;
  std::vector<int32_t> timesteps;
  int64_t iteration;                                    // n
};

namespace {

int64_t last_iteration(const ca_sched* s) {
  return int64_t(s->lag) * (s->n_blocks - 1) + int64_t(s->timesteps.size()) - 1;
}

// blocks in flight in iteration n: first (oldest) block and count
void batch_range(const ca_sched* s, int64_t n, int64_t* first, int32_t* count) {
  const int64_t nT = int64_t(s->timesteps.size());
  // n - lag*j <= nT - 1  <=>  j >= (n - nT + 1) / lag (rounded up);  n - lag*j >= 0  <=>  j <= n / lag
  int64_t lo = n - nT + 1 <= 0 ? 0 : (n - nT + 1 + s->lag - 1) / s->lag;
  int64_t hi = n / s->lag;
  if (hi > s->n_blocks - 1) hi = s->n_blocks - 1;
  *first = lo;
  *count = hi >= lo ? int32_t(hi - lo + 1) : 0;
}

}  // namespace

extern "C" {

int32_t ca_sched_create_lagged(int64_t n_blocks, const int32_t* timesteps, int32_t n_timesteps, int32_t lag,
                               ca_sched** out) {
  if (!out || !timesteps || n_timesteps < 2 || n_blocks < 1 || lag < 1 || lag > n_timesteps) return CA_EINVAL;
  ca_sched* s = new (std::nothrow) ca_sched();
  if (!s) return CA_EINVAL;
  s->n_blocks = n_blocks;
  s->lag = lag;
  s->timesteps.assign(timesteps, timesteps + n_timesteps);
  s->iteration = 0;
  *out = s;
  return CA_OK;
}

int32_t ca_sched_create(int64_t n_blocks, int32_t n_parallel, const int32_t* timesteps, int32_t n_timesteps,
                        ca_sched** out) {
  if (!out || !timesteps || n_timesteps < 2 || n_parallel < 1 || n_blocks < 1) return CA_EINVAL;
  if (n_parallel != n_timesteps || n_blocks < n_parallel) return CA_EUNSUPPORTED;
  return ca_sched_create_lagged(n_blocks, timesteps, n_timesteps, 1, out);
}

int32_t ca_sched_destroy(ca_sched* s) {
  if (!s) return CA_EINVAL;
  delete s;
  return CA_OK;
}

int32_t ca_sched_batch(const ca_sched* s, ca_sched_entry* out, int32_t cap, int32_t* n_out) {
  if (!s || !n_out || cap < 0 || (cap > 0 && !out)) return CA_EINVAL;
  if (s->iteration > last_iteration(s)) {               // rollout complete
    *n_out = 0;
    return CA_OK;
  }
  int64_t first;
  int32_t n;
  batch_range(s, s->iteration, &first, &n);
  if (cap < n) return CA_EINVAL;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t idx = int32_t(s->iteration - int64_t(s->lag) * (first + i));
    out[i].block_id = first + i;
    out[i].timestep_index = idx;
    out[i].timestep = s->timesteps[idx];
  }
  *n_out = n;
  return CA_OK;
}

int32_t ca_sched_advance(ca_sched* s, int64_t* emitted_block, int64_t* completed_block) {
  if (!s) return CA_EINVAL;
  if (s->iteration > last_iteration(s)) return CA_ESTATE;
  const int32_t nT = int32_t(s->timesteps.size());
  int64_t first;
  int32_t n;
  batch_range(s, s->iteration, &first, &n);
  int64_t emitted = -1, completed = -1;
  for (int32_t i = 0; i < n; ++i) {
    const int64_t idx = s->iteration - int64_t(s->lag) * (first + i);
    if (idx == nT - 2) emitted = first + i;             // ran at t0: its prediction is the output
    if (idx == nT - 1) completed = first + i;           // ran at tc
  }
  s->iteration += 1;
  if (emitted_block) *emitted_block = emitted;
  if (completed_block) *completed_block = completed;
  return CA_OK;
}

int32_t ca_sched_state(const ca_sched* s, int64_t* b, int32_t* tau, int32_t* d, int64_t* iteration) {
  if (!s) return CA_EINVAL;
  int64_t first = s->n_blocks;
  int32_t n = 0;
  if (s->iteration <= last_iteration(s)) batch_range(s, s->iteration, &first, &n);
  if (b) *b = first;
  if (tau) *tau = n ? int32_t(s->iteration - int64_t(s->lag) * first) : int32_t(s->timesteps.size()) - 1;
  if (d) *d = n - 1;
  if (iteration) *iteration = s->iteration;
  return CA_OK;
}

}  // extern "C"
