// Host-side cascade scheduler: the control flow of Algorithm 1 ("Multi-GPU Inference with Block
// Cascading"), integers only.  State (b, tau, d): primary block, timestep index of the primary
// block, cascade depth.  An iteration forwards blocks b .. b+min(d, G-1), block b+i at timestep
// T[tau - i]; afterwards a block that ran at t0 (the second-to-last entry of T) is emitted, a block
// that ran at tc (the last entry) is complete, and the state advances as in the listing.
//
// The listing is self-consistent only when the number of parallel blocks G equals the number of
// timesteps (otherwise a new block would enter in the middle of the schedule), and it ramps the
// depth past the last block when there are fewer blocks than G; both cases are rejected here.
#include <new>
#include <vector>

#include "cascade_attn.h"

struct ca_sched {
  int64_t n_blocks;
  int32_t n_parallel;
  std::vector<int32_t> timesteps;
  int64_t b;
  int32_t tau, d;
  int64_t iteration;
};

extern "C" {

int32_t ca_sched_create(int64_t n_blocks, int32_t n_parallel, const int32_t* timesteps,
                        int32_t n_timesteps, ca_sched** out) {
  if (!out || !timesteps || n_timesteps < 2 || n_parallel < 1 || n_blocks < 1) return CA_EINVAL;
  if (n_parallel != n_timesteps || n_blocks < n_parallel) return CA_EUNSUPPORTED;
  ca_sched* s = new (std::nothrow) ca_sched();
  if (!s) return CA_EINVAL;
  s->n_blocks = n_blocks;
  s->n_parallel = n_parallel;
  s->timesteps.assign(timesteps, timesteps + n_timesteps);
  s->b = 0;
  s->tau = 0;
  s->d = 0;
  s->iteration = 0;
  *out = s;
  return CA_OK;
}

int32_t ca_sched_destroy(ca_sched* s) {
  if (!s) return CA_EINVAL;
  delete s;
  return CA_OK;
}

int32_t ca_sched_batch(const ca_sched* s, ca_sched_entry* out, int32_t cap, int32_t* n_out) {
  if (!s || !n_out || cap < 0 || (cap > 0 && !out)) return CA_EINVAL;
  if (s->d < 0) {                       // rollout complete
    *n_out = 0;
    return CA_OK;
  }
  const int32_t n = (s->d < s->n_parallel - 1 ? s->d : s->n_parallel - 1) + 1;
  if (cap < n) return CA_EINVAL;
  for (int32_t i = 0; i < n; ++i) {
    out[i].block_id = s->b + i;
    out[i].timestep_index = s->tau - i;
    out[i].timestep = s->timesteps[s->tau - i];
  }
  *n_out = n;
  return CA_OK;
}

int32_t ca_sched_advance(ca_sched* s, int64_t* emitted_block, int64_t* completed_block) {
  if (!s) return CA_EINVAL;
  if (s->d < 0) return CA_ESTATE;
  const int32_t nT = int32_t(s->timesteps.size());
  const int32_t n = (s->d < s->n_parallel - 1 ? s->d : s->n_parallel - 1) + 1;
  int64_t emitted = -1, completed = -1;
  for (int32_t j = 0; j < n; ++j)
    if (s->tau - j == nT - 2) emitted = s->b + j;      // ran at t0: its prediction is the output
  if (s->tau == nT - 1) {                               // block b completed tc
    completed = s->b;
    s->b += 1;
    if (s->b + s->d >= s->n_blocks) s->d -= 1;
  } else {
    s->d = s->d + 1 < s->n_parallel - 1 ? s->d + 1 : s->n_parallel - 1;
    s->tau += 1;
  }
  s->iteration += 1;
  if (emitted_block) *emitted_block = emitted;
  if (completed_block) *completed_block = completed;
  return CA_OK;
}

int32_t ca_sched_state(const ca_sched* s, int64_t* b, int32_t* tau, int32_t* d, int64_t* iteration) {
  if (!s) return CA_EINVAL;
  if (b) *b = s->b;
  if (tau) *tau = s->tau;
  if (d) *d = s->d;
  if (iteration) *iteration = s->iteration;
  return CA_OK;
}

}  // extern "C"
