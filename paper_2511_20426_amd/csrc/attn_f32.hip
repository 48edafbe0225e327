// fp32 block-cascaded attention for the small fp32 configuration (head_dim 32/64/128).
//
// One thread owns one query row and walks the visible KV pages with a running-max softmax;
// all lanes of a wave read the same K/V row at a time, which the hardware serves as a
// broadcast.  This path exists for exactness on small problems, not for speed: the bf16 MFMA
// kernel is the throughput path.
//
// Visibility per block pair follows Sec. 3.1 (a block is bidirectional inside), Sec. 3.3
// (cached blocks visible to all) and Sec. 3.4 / 4.2 (bidirectional or block-causal cascade).
#include <hip/hip_runtime.h>

#include "ca_internal.hpp"

namespace ca {
namespace {

template <int D>
__global__ __launch_bounds__(64) void attn_f32_kernel(AttnPlan p, const float* __restrict__ q,
                                                      float* __restrict__ out,
                                                      const float* __restrict__ pool) {
  const int L = p.block_tokens;
  const int h = blockIdx.y;
  const int qb = blockIdx.z;                                  // in-flight (query) block
  const int r = blockIdx.x * 64 + threadIdx.x;                // row inside the block
  const bool live = r < L;
  const int64_t row = int64_t(qb) * L + (live ? r : 0);
  const float* qp = q + (row * p.heads + h) * D;
  float qv[D], acc[D];
#pragma unroll
  for (int d = 0; d < D; ++d) { qv[d] = qp[d]; acc[d] = 0.f; }
  const float scale = 1.0f / sqrtf(float(D));
  float m = -INFINITY, l = 0.f;
  const size_t page_elems = size_t(p.page_tokens) * D;
  const int nvis = p.n_vis[qb];
  for (int kb = 0; kb < nvis; ++kb) {
    const int slot = p.kv_slot[kb];
    for (int pg = 0; pg < p.pages_per_block; ++pg) {
      const size_t pair = (size_t(slot) * p.pages_per_block + pg) * p.heads + h;
      const float* kp = pool + pair * 2 * page_elems;
      const float* vp = kp + page_elems;
      const int valid = min(p.page_tokens, L - pg * p.page_tokens);
      for (int t = 0; t < valid; ++t) {
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) s = fmaf(qv[d], kp[size_t(t) * D + d], s);
        s *= scale;
        const float m_new = fmaxf(m, s);
        const float alpha = expf(m - m_new);      // 0 on the first key (m = -inf)
        const float w = expf(s - m_new);
        l = l * alpha + w;
#pragma unroll
        for (int d = 0; d < D; ++d) acc[d] = fmaf(acc[d], alpha, w * vp[size_t(t) * D + d]);
        m = m_new;
      }
    }
  }
  if (live) {
    const float inv = 1.0f / l;
    float* op = out + (row * p.heads + h) * D;
#pragma unroll
    for (int d = 0; d < D; ++d) op[d] = acc[d] * inv;
  }
}

}  // namespace

int32_t launch_attn_f32(const AttnPlan& p, const void* q, void* out, const void* pool, void* stream) {
  const dim3 grid((unsigned)((p.block_tokens + 63) / 64), (unsigned)p.heads, (unsigned)p.n_q_blocks);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const float* qf = static_cast<const float*>(q);
  float* of = static_cast<float*>(out);
  const float* pf = static_cast<const float*>(pool);
  switch (p.head_dim) {
    case 32: hipLaunchKernelGGL(attn_f32_kernel<32>, grid, dim3(64), 0, s, p, qf, of, pf); break;
    case 64: hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(64), 0, s, p, qf, of, pf); break;
    case 128: hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(64), 0, s, p, qf, of, pf); break;
    default: return CA_EUNSUPPORTED;
  }
  return finish_launch("attn_f32.hip");
}

}  // namespace ca
