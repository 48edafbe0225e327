// 3-axis rotary embedding and the fused "rotate K + store K/V pages" cache write (gfx950).
//
// Both are HBM-bound: every element is read once and written once.  The trigonometry is
// shared by all heads of a token, so a thread evaluates sin/cos (in fp64, once) for the
// pairs it owns and reuses them across its head loop; rotation itself is fp32 with a single
// round-to-nearest-even to the storage type.
//
// The paper publishes each in-flight block's K/V to a shared pool at every self-attention
// layer (Sec. 3.3); rotary embedding is the Wan-family convention (see cascade_attn.h).
#include <hip/hip_runtime.h>

#include <atomic>

#include <cstdio>

#include "ca_internal.hpp"

namespace ca {
namespace {

#include "rope_device.hpp"

// ----------------------------------------------------------------------------- generic path
// One thread owns 4 consecutive pairs (8 elements) of one token and walks a range of heads; the 64
// lanes of a wave cover one token: 64/chunks neighbouring heads x all chunks, i.e. up to 1 KB of
// contiguous memory per load when heads are adjacent in memory.
// MODE 0: y[token][head][dim] (rope3d_apply).  MODE 1: K/V pages of the fp32 pool layout
// (row-major [token][dim] pages), V copied unrotated.
struct GenericArgs {
  const void* x;        // MODE 0: input; MODE 1: K
  const void* v;        // MODE 1: V
  void* y;              // MODE 0: output; MODE 1: pool
  int64_t n_tokens, first_frame, tok_stride, head_stride;
  int64_t y_tok_stride, y_head_stride;   // MODE 0: strides of the output
  int32_t heads_per_group;
  // MODE 1 only: n_tokens covers whole pages, tokens >= valid_tokens are stored as zeros
  int32_t page_tokens, pages_per_block, slot, valid_tokens;
};

template <typename T, int MODE>
__global__ __launch_bounds__(256) void rope_generic_kernel(RopeGeom g, GenericArgs a) {
  const int chunks = g.head_dim / 8;              // 4, 8 or 16
  const int head_slots = 64 / chunks;             // heads a wave touches per load
  const int64_t n = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (n >= a.n_tokens) return;
  const int lane = threadIdx.x & 63;
  const int c8 = lane % chunks;
  const int hs = lane / chunks;
  const bool pad = MODE == 1 && n >= a.valid_tokens;
  const TokenPos p = token_pos(pad ? 0 : n, a.first_frame, g.grid_h, g.grid_w);
  float cs[4], sn[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) pair_cs<sizeof(T) == 4>(g, p, c8 * 4 + j, &cs[j], &sn[j]);
  const int h0 = blockIdx.y * a.heads_per_group;
  const int h1 = min(h0 + a.heads_per_group, g.heads);
  const T* x = static_cast<const T*>(a.x);
  for (int h = h0 + hs; h < h1; h += head_slots) {
    const int64_t src = n * a.tok_stride + int64_t(h) * a.head_stride + c8 * 8;
    Vec8<T> e, w;
#pragma unroll
    for (int j = 0; j < 8; ++j) e.v[j] = w.v[j] = 0.f;
    if (!pad) {
      e.load(x + src);
      rotate8(e, cs, sn);
    }
    if (MODE == 0) {
      e.store(static_cast<T*>(a.y) + n * a.y_tok_stride + int64_t(h) * a.y_head_stride + c8 * 8);
    } else {
      const int64_t page = n / a.page_tokens, row = n % a.page_tokens;
      const int64_t page_elems = int64_t(a.page_tokens) * g.head_dim;
      const int64_t pair = (int64_t(a.slot) * a.pages_per_block + page) * g.heads + h;
      T* kdst = static_cast<T*>(a.y) + pair * 2 * page_elems + row * g.head_dim + c8 * 8;
      e.store(kdst);
      if (!pad) w.load(static_cast<const T*>(a.v) + src);
      w.store(kdst + page_elems);
    }
  }
}

// ----------------------------------------------------------------------------- bf16 paged write
// head_dim 128, 128-token pages.  One workgroup writes one page for a group of heads.
// K page: row = token, sixteen 16-byte chunks, chunk c kept at position c ^ (row & 15).
// V page: row = dim, chunk c = eight tokens in MFMA hand-over order, same swizzle.
// V goes through LDS to be transposed; rows of 65 dwords keep the column reads conflict-free.
constexpr int kPage = 128;
constexpr int kVRowWords = 65;

struct PagedBlock {            // one block of a launch (grid.z picks it)
  const uint16_t* k;
  const uint16_t* v;
  int64_t first_frame;
  int32_t slot;
};

struct PagedBatch {
  PagedBlock b[kMaxInflight];
  uint8_t* pool;
  int64_t tok_stride, head_stride;
  int32_t block_tokens, pages_per_block, heads_per_group;
  TrigTable tab;               // n_f == 0: no table (geometry too large for LDS), evaluate per thread
};

struct PagedArgs {             // what the kernel body works with: the batch's entry for this workgroup
  const uint16_t* k;
  const uint16_t* v;
  uint8_t* pool;
  int64_t tok_stride, head_stride, first_frame;
  int32_t block_tokens, pages_per_block, slot, heads_per_group;
  TrigTable tab;
};

__global__ __launch_bounds__(256) void cache_write_bf16_kernel(RopeGeom g, PagedBatch batch) {
  PagedArgs a;
  {
    const PagedBlock& blk = batch.b[blockIdx.z];
    a.k = blk.k; a.v = blk.v; a.first_frame = blk.first_frame; a.slot = blk.slot;
    a.pool = batch.pool; a.tok_stride = batch.tok_stride; a.head_stride = batch.head_stride;
    a.block_tokens = batch.block_tokens; a.pages_per_block = batch.pages_per_block;
    a.heads_per_group = batch.heads_per_group; a.tab = batch.tab;
  }
  __shared__ uint32_t vt[kPage * kVRowWords];
  extern __shared__ float2 trig[];   // [n_f][pairs_t] then [n_y][pairs_h] then [n_x][pairs_w]
  const int t = threadIdx.x;
  const int page = blockIdx.x;
  const int c = t & 15;              // chunk owned by this thread (K: dims 8c..8c+7; V: 8 tokens)
  const int r0 = t >> 4;             // first row; rows r0, r0+16, ..., r0+112
  const int tok0 = page * kPage;

  // cos/sin of this thread's 4 pairs at its 8 tokens
  float cs[8][4], sn[8][4];
  if (a.tab.n_f > 0) {
    const TrigLayout lay = trig_layout(g, a.tab, tok0, a.block_tokens, a.first_frame);
    trig_fill(g, lay, trig, t, 256);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int n = tok0 + r0 + 16 * i;
      const TokenPos p = token_pos(min(n, a.block_tokens - 1), a.first_frame, g.grid_h, g.grid_w);
      trig_pick(g, lay, trig, p, c, cs[i], sn[i]);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int n = tok0 + r0 + 16 * i;
      const TokenPos p = token_pos(min(n, a.block_tokens - 1), a.first_frame, g.grid_h, g.grid_w);
#pragma unroll
      for (int j = 0; j < 4; ++j) pair_cs<false>(g, p, c * 4 + j, &cs[i][j], &sn[i][j]);
    }
  }

  const int h0 = blockIdx.y * a.heads_per_group;
  const int h1 = min(h0 + a.heads_per_group, g.heads);
  for (int h = h0; h < h1; ++h) {
    const int64_t pair = (int64_t(a.slot) * a.pages_per_block + page) * g.heads + h;
    uint8_t* kpage = a.pool + pair * (2 * kPage * 128 * 2);
    uint8_t* vpage = kpage + kPage * 128 * 2;
    // ---- K: rotate and store swizzled; V: stage into LDS
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = r0 + 16 * i;
      const int n = tok0 + r;
      U4 kk = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
      if (n < a.block_tokens) {
        const int64_t src = int64_t(n) * a.tok_stride + int64_t(h) * a.head_stride + c * 8;
        Vec8<uint16_t> e;
        e.load(a.k + src);
        rotate8(e, cs[i], sn[i]);
        kk.x = pack_bf16(e.v[0], e.v[1]); kk.y = pack_bf16(e.v[2], e.v[3]);
        kk.z = pack_bf16(e.v[4], e.v[5]); kk.w = pack_bf16(e.v[6], e.v[7]);
        vv = load_once(a.v + src);
      }
      *reinterpret_cast<U4*>(kpage + r * 256 + ((c ^ (r & 15)) << 4)) = kk;
      uint32_t* row = vt + r * kVRowWords + c * 4;
      row[0] = vv.x; row[1] = vv.y; row[2] = vv.z; row[3] = vv.w;
    }
    __syncthreads();
    // ---- V: thread builds chunk c of dim rows r0 + 16 i: tokens 16*(c/2) + perm[8*(c%2) + e]
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int d = r0 + 16 * i;
      const int tb = 16 * (c >> 1) + 4 * (c & 1);     // tokens tb..tb+3 and tb+8..tb+11
      uint32_t e[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int tok = tb + (j & 3) + 8 * (j >> 2);
        const uint32_t w = vt[tok * kVRowWords + (d >> 1)];
        e[j] = (d & 1) ? (w >> 16) : (w & 0xffffu);
      }
      U4 o;
      o.x = e[0] | (e[1] << 16); o.y = e[2] | (e[3] << 16);
      o.z = e[4] | (e[5] << 16); o.w = e[6] | (e[7] << 16);
      *reinterpret_cast<U4*>(vpage + d * 256 + ((c ^ (d & 15)) << 4)) = o;
    }
    __syncthreads();
  }
}

}  // namespace

namespace {
thread_local char g_last_error[256] = "";
}

int32_t finish_launch(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return CA_OK;
  snprintf(g_last_error, sizeof(g_last_error), "%s: %s", what, hipGetErrorString(e));
  return CA_EDEVICE;
}

int32_t device_failure(const char* what, int hip_error) {
  (void)hipGetLastError();
  snprintf(g_last_error, sizeof(g_last_error), "%s: %s", what, hipGetErrorString(static_cast<hipError_t>(hip_error)));
  return CA_EDEVICE;
}

const char* last_device_error() { return g_last_error; }

namespace {
std::atomic<int> g_cu_count[kMaxDevices];
std::atomic<int> g_lds_set[4][kMaxDevices];
}  // namespace

int32_t device_cu_count(int* n_cu) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return finish_launch("hipGetDevice");
  const bool cached = dev >= 0 && dev < kMaxDevices;
  int n = cached ? g_cu_count[dev].load(std::memory_order_relaxed) : 0;
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      return finish_launch("hipDeviceGetAttribute");
    if (n <= 0) return CA_EDEVICE;
    if (cached) g_cu_count[dev].store(n, std::memory_order_relaxed);
  }
  *n_cu = n;
  return CA_OK;
}

int32_t ensure_dynamic_lds(const void* kernel, int bytes, int slot) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return finish_launch("hipGetDevice");
  const bool cached = dev >= 0 && dev < kMaxDevices;
  if (cached && g_lds_set[slot][dev].load(std::memory_order_relaxed) == bytes) return CA_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
    return finish_launch("hipFuncSetAttribute");
  if (cached) g_lds_set[slot][dev].store(bytes, std::memory_order_relaxed);
  return CA_OK;
}

int32_t launch_rope_apply(const RopeGeom& g, int dtype, const void* x, void* y, int64_t n_tokens,
                          int64_t first_frame, int64_t tok_stride, int64_t head_stride,
                          int64_t y_tok_stride, int64_t y_head_stride, void* stream) {
  if (n_tokens == 0) return CA_OK;
  GenericArgs a{};
  a.x = x; a.v = nullptr; a.y = y;
  a.n_tokens = n_tokens; a.first_frame = first_frame;
  a.tok_stride = tok_stride; a.head_stride = head_stride;
  a.y_tok_stride = y_tok_stride; a.y_head_stride = y_head_stride;
  const int64_t gx = (n_tokens + 3) / 4;           // one wave per token, four per workgroup
  if (gx > 0x7fffffff) return CA_EINVAL;
  // enough workgroups to fill 256 CUs several times over, few enough to amortise the trig
  int groups = 1;
  while (gx * groups < 2048 && groups < g.heads) groups *= 2;
  groups = groups > g.heads ? g.heads : groups;
  a.heads_per_group = (g.heads + groups - 1) / groups;
  const dim3 grid((unsigned)gx, (unsigned)((g.heads + a.heads_per_group - 1) / a.heads_per_group));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == CA_BF16)
    hipLaunchKernelGGL((rope_generic_kernel<uint16_t, 0>), grid, dim3(256), 0, s, g, a);
  else
    hipLaunchKernelGGL((rope_generic_kernel<float, 0>), grid, dim3(256), 0, s, g, a);
  return finish_launch("rope_cache.hip");
}

int32_t launch_cache_write(const RopeGeom& g, int dtype, int32_t n_blocks, const void* const* k,
                           const void* const* v, int64_t tok_stride, int64_t head_stride,
                           const int64_t* first_frame, int32_t block_tokens, int32_t page_tokens,
                           int32_t pages_per_block, const int32_t* slot, void* pool, void* stream) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (n_blocks < 1 || n_blocks > kMaxInflight) return CA_EINVAL;
  if (dtype == CA_BF16) {
    if (g.head_dim != 128 || page_tokens != kPage) return CA_EUNSUPPORTED;
    PagedBatch a{};
    for (int i = 0; i < n_blocks; ++i) {
      a.b[i].k = static_cast<const uint16_t*>(k[i]);
      a.b[i].v = static_cast<const uint16_t*>(v[i]);
      a.b[i].first_frame = first_frame[i];
      a.b[i].slot = slot[i];
    }
    a.pool = static_cast<uint8_t*>(pool);
    a.tok_stride = tok_stride; a.head_stride = head_stride;
    a.block_tokens = block_tokens; a.pages_per_block = pages_per_block;
    int groups = 1;
    while (pages_per_block * n_blocks * groups < 1024 && groups < g.heads) groups *= 2;
    groups = groups > g.heads ? g.heads : groups;
    a.heads_per_group = (g.heads + groups - 1) / groups;
    const dim3 grid((unsigned)pages_per_block,
                    (unsigned)((g.heads + a.heads_per_group - 1) / a.heads_per_group), (unsigned)n_blocks);
    size_t tab_bytes = 0;
    const TrigTable tab = trig_table_for(g, kPage, 16384, &tab_bytes);
    a.tab = tab;
    hipLaunchKernelGGL(cache_write_bf16_kernel, grid, dim3(256), tab_bytes, s, g, a);
  } else {
    for (int i = 0; i < n_blocks; ++i) {           // the fp32 path is for tiny cases: one launch per block
      GenericArgs a{};
      a.x = k[i]; a.v = v[i]; a.y = pool;
      a.n_tokens = int64_t(pages_per_block) * page_tokens; a.first_frame = first_frame[i];
      a.valid_tokens = block_tokens;
      a.tok_stride = tok_stride; a.head_stride = head_stride;
      a.page_tokens = page_tokens; a.pages_per_block = pages_per_block; a.slot = slot[i];
      a.heads_per_group = g.heads;
      const dim3 grid((unsigned)((a.n_tokens + 3) / 4), 1);
      hipLaunchKernelGGL((rope_generic_kernel<float, 1>), grid, dim3(256), 0, s, g, a);
    }
  }
  return finish_launch("rope_cache.hip");
}

}  // namespace ca
