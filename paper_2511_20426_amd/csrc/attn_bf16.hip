// bf16 block-cascaded attention on the gfx950 matrix cores (head_dim 128, 128-token pages).
//
// What it computes: for every in-flight query block, softmax(Q K^T / sqrt(D)) V over the
// pages of the KV blocks that block may see -- the clean cache plus the in-flight blocks,
// all of them (bidirectional cascade, Sec. 3.4) or those not later than itself (block-causal,
// Sec. 3.2 / 4.2).  Visibility is per block pair, so masking is "walk only the visible pages":
// pages of invisible blocks are never loaded.
//
// Shape of the kernel
//   workgroup = 4 waves, one per SIMD; a wave owns 64 query rows (two 32-wide MFMA column
//   tiles), a workgroup 256 rows of one head.  K/V pages (32 KB + 32 KB) are streamed
//   through a double-buffered LDS ring and shared by the four waves.
//   S^T = K Q^T   : v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q (registers).
//                   In the 32x32 accumulator layout a lane then holds 16 of the 32 keys of ONE
//                   query, so the row max / row sum need a single cross-lane step (lane ^ 32).
//   O^T += V^T P^T: A = V^T rows from LDS, B = P^T straight from the S^T accumulator
//                   registers (rounded to bf16).  V pages are stored transposed and with the
//                   key order the accumulator hands over, so no data movement is needed
//                   between the two products (see cascade_attn.h for the page format).
//   Softmax is the running-max form in base 2: p = exp2(s*c - m), c = log2(e)/sqrt(D); the
//   accumulator is rescaled only on iterations where some row max of the wave grew.
//   The 256-byte page rows are stored with their 16-byte chunks XOR-swizzled by (row & 15),
//   which makes every ds_read_b128 of an MFMA operand bank-conflict free.
//   Workgroups are numbered so that the eight XCDs each take a contiguous range of
//   (head, row tile) work: workgroups running together on an XCD stream the same head's pages
//   and share them in that XCD's L2.
#include <hip/hip_runtime.h>

#include "ca_internal.hpp"

namespace ca {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kPageBytes = 128 * 128 * 2;       // one K or V page
constexpr int kPairBytes = 2 * kPageBytes;      // K page followed by V page
constexpr int kRowsPerWg = 256;
constexpr int kMaxSeg = kMaxInflight;

struct AttnArgs {
  const uint16_t* q;
  uint16_t* o;
  const uint8_t* pool;
  int32_t heads, pages_per_block, last_valid;
  int32_t n_seg;                       // query segments: rows that share one visible prefix
  int32_t seg_row0[kMaxSeg], seg_rows[kMaxSeg], seg_nvis[kMaxSeg], seg_tile0[kMaxSeg + 1];
  int32_t kv_slot[kMaxKvBlocks];
  int32_t tiles_per_head, total_work, work_per_xcd;
  float c;                             // log2(e) / sqrt(head_dim)
};

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(uint32_t, b);
}

// value of the partner lane (lane ^ 32)
__device__ __forceinline__ float other_half(float x) {
  return __shfl_xor(x, 32, 64);
}

__device__ __forceinline__ bf16x8 lds_read16(const uint8_t* lds, uint32_t off) {
  return *reinterpret_cast<const bf16x8*>(lds + off);
}

__global__ __launch_bounds__(256, 1) void attn_bf16_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, hi = lane >> 5, sw = lane & 15;

  // ---- which (head, row tile): XCD x takes work items [x*work_per_xcd, (x+1)*work_per_xcd)
  const int xcd = blockIdx.x & 7, nth = blockIdx.x >> 3;
  const int work = xcd * a.work_per_xcd + nth;
  if (nth >= a.work_per_xcd || work >= a.total_work) return;
  const int h = work / a.tiles_per_head;
  const int tile = work - h * a.tiles_per_head;
  int seg = 0;
  while (seg + 1 < a.n_seg && tile >= a.seg_tile0[seg + 1]) ++seg;
  const int row0 = a.seg_row0[seg] + (tile - a.seg_tile0[seg]) * kRowsPerWg;
  const int rows_end = a.seg_row0[seg] + a.seg_rows[seg];
  const int n_iter = a.seg_nvis[seg] * a.pages_per_block;

  // ---- Q fragments: B operand, lane holds dims 16ks + 8hi .. +7 of query (l31) per column tile
  bf16x8 qf[2][8];
  int qrow[2];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    qrow[nt] = row0 + wave * 64 + nt * 32 + l31;
    const bool ok = qrow[nt] < rows_end;
    const uint16_t* qp = a.q + (int64_t(ok ? qrow[nt] : row0) * a.heads + h) * 128 + hi * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      u32x4 v = *reinterpret_cast<const u32x4*>(qp + ks * 16);
      if (!ok) v = u32x4{0, 0, 0, 0};
      qf[nt][ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  // ---- LDS operand offsets (swizzled chunk = logical chunk ^ (row & 15), row & 15 == lane & 15)
  uint32_t koff[8], voff[4][2];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) koff[ks] = l31 * 256 + (((2 * ks + hi) ^ sw) << 4);
#pragma unroll
  for (int sub = 0; sub < 4; ++sub)
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
      voff[sub][kk] = kPageBytes + l31 * 256 + (((4 * sub + 2 * kk + hi) ^ sw) << 4);

  f32x16 oacc[4][2];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[mt][nt][i] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY};   // running max of s*c
  float l_run[2] = {0.f, 0.f};               // this lane's share of the running sum

  auto page_ptr = [&](int it) -> const uint8_t* {
    const int kb = it / a.pages_per_block, pg = it - kb * a.pages_per_block;
    const int64_t pair = (int64_t(a.kv_slot[kb]) * a.pages_per_block + pg) * a.heads + h;
    return a.pool + pair * kPairBytes;
  };

  // ---- prologue: page 0 -> LDS stage 0
  u32x4 st[16];
  {
    const uint8_t* src = page_ptr(0);
#pragma unroll
    for (int i = 0; i < 16; ++i) st[i] = *reinterpret_cast<const u32x4*>(src + (i * 256 + tid) * 16);
#pragma unroll
    for (int i = 0; i < 16; ++i) *reinterpret_cast<u32x4*>(lds + (i * 256 + tid) * 16) = st[i];
  }
  __syncthreads();

  for (int it = 0; it < n_iter; ++it) {
    const uint8_t* cur = lds + (it & 1) * kPairBytes;
    const bool more = it + 1 < n_iter;
    if (more) {
      const uint8_t* src = page_ptr(it + 1);
#pragma unroll
      for (int i = 0; i < 16; ++i) st[i] = *reinterpret_cast<const u32x4*>(src + (i * 256 + tid) * 16);
    }
    const int pg = it % a.pages_per_block;
    const int valid = pg == a.pages_per_block - 1 ? a.last_valid : 128;

#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      if (sub * 32 < valid) {
        // ---- S^T tile: 32 keys x (2 x 32) queries
        f32x16 s[2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int i = 0; i < 16; ++i) s[nt][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const bf16x8 kf = lds_read16(cur, sub * 8192 + koff[ks]);
          s[0] = mfma(kf, qf[0][ks], s[0]);
          s[1] = mfma(kf, qf[1][ks], s[1]);
        }
        if (valid < sub * 32 + 32) {       // ragged last page: keys past the block end
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = sub * 32 + 8 * (i >> 2) + 4 * hi + (i & 3);
            if (key >= valid) { s[0][i] = -INFINITY; s[1][i] = -INFINITY; }
          }
        }
        // ---- running-max softmax, base 2
        float m_new[2];
        bool grew = false;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          float mx = s[nt][0];
#pragma unroll
          for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[nt][i]);
          mx = fmaxf(mx, other_half(mx));
          m_new[nt] = fmaxf(m_run[nt], mx * a.c);
          grew |= m_new[nt] > m_run[nt];
        }
        if (__builtin_amdgcn_ballot_w64(grew) != 0) {
#pragma unroll
          for (int nt = 0; nt < 2; ++nt) {
            const float alpha = __builtin_amdgcn_exp2f(m_run[nt] - m_new[nt]);
            l_run[nt] *= alpha;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
              for (int i = 0; i < 16; ++i) oacc[mt][nt][i] *= alpha;
            m_run[nt] = m_new[nt];
          }
        }
        bf16x8 pb[2][2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          float p[16];
          float sum = 0.f;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            p[i] = __builtin_amdgcn_exp2f(fmaf(s[nt][i], a.c, -m_run[nt]));
            sum += p[i];
          }
          l_run[nt] += sum;
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) {
            u32x4 w;
            w[0] = pack2(p[8 * kk + 0], p[8 * kk + 1]);
            w[1] = pack2(p[8 * kk + 2], p[8 * kk + 3]);
            w[2] = pack2(p[8 * kk + 4], p[8 * kk + 5]);
            w[3] = pack2(p[8 * kk + 6], p[8 * kk + 7]);
            pb[nt][kk] = __builtin_bit_cast(bf16x8, w);
          }
        }
        // ---- O^T += V^T P^T
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) {
            const bf16x8 vf = lds_read16(cur, mt * 8192 + voff[sub][kk]);
            oacc[mt][0] = mfma(vf, pb[0][kk], oacc[mt][0]);
            oacc[mt][1] = mfma(vf, pb[1][kk], oacc[mt][1]);
          }
      }
    }

    if (more) {
      uint8_t* nxt = lds + ((it + 1) & 1) * kPairBytes;
#pragma unroll
      for (int i = 0; i < 16; ++i) *reinterpret_cast<u32x4*>(nxt + (i * 256 + tid) * 16) = st[i];
    }
    __syncthreads();
  }

  // ---- normalise and store: lane holds, for its query, dims 32mt + 8(i/4) + 4hi + (i%4)
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float l_tot = l_run[nt] + other_half(l_run[nt]);
    const float inv = 1.0f / l_tot;
    if (qrow[nt] < rows_end) {
      uint16_t* op = a.o + (int64_t(qrow[nt]) * a.heads + h) * 128 + 4 * hi;
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 w;
          w[0] = pack2(oacc[mt][nt][4 * g + 0] * inv, oacc[mt][nt][4 * g + 1] * inv);
          w[1] = pack2(oacc[mt][nt][4 * g + 2] * inv, oacc[mt][nt][4 * g + 3] * inv);
          *reinterpret_cast<u32x2*>(op + 32 * mt + 8 * g) = w;
        }
    }
  }
}

}  // namespace

int32_t attn_bf16_variant_ok(int variant) { return variant == 0 ? CA_OK : CA_EINVAL; }

int32_t launch_attn_bf16(const AttnPlan& p, int variant, const void* q, void* out, const void* pool,
                         void* stream) {
  if (p.head_dim != 128 || p.page_tokens != 128) return CA_EUNSUPPORTED;
  if (attn_bf16_variant_ok(variant) != CA_OK) return CA_EINVAL;
  AttnArgs a{};
  a.q = static_cast<const uint16_t*>(q);
  a.o = static_cast<uint16_t*>(out);
  a.pool = static_cast<const uint8_t*>(pool);
  a.heads = p.heads;
  a.pages_per_block = p.pages_per_block;
  a.last_valid = p.block_tokens - (p.pages_per_block - 1) * 128;
  for (int i = 0; i < p.n_kv; ++i) a.kv_slot[i] = p.kv_slot[i];
  // Query segments: rows sharing one visible prefix are tiled together.  A bidirectional
  // cascade is one segment; block-causal gives one segment per in-flight block.
  int tiles = 0;
  if (p.uniform) {
    a.n_seg = 1;
    a.seg_row0[0] = 0;
    a.seg_rows[0] = p.n_q_blocks * p.block_tokens;
    a.seg_nvis[0] = p.n_vis[0];
    a.seg_tile0[0] = 0;
    tiles = (a.seg_rows[0] + kRowsPerWg - 1) / kRowsPerWg;
    a.seg_tile0[1] = tiles;
  } else {
    // heaviest segment (latest block, longest prefix) first, so the tail of the launch is light
    a.n_seg = p.n_q_blocks;
    for (int j = 0; j < p.n_q_blocks; ++j) {
      const int i = p.n_q_blocks - 1 - j;
      a.seg_row0[j] = i * p.block_tokens;
      a.seg_rows[j] = p.block_tokens;
      a.seg_nvis[j] = p.n_vis[i];
      a.seg_tile0[j] = tiles;
      tiles += (p.block_tokens + kRowsPerWg - 1) / kRowsPerWg;
    }
    a.seg_tile0[p.n_q_blocks] = tiles;
  }
  a.tiles_per_head = tiles;
  a.total_work = tiles * p.heads;
  a.work_per_xcd = (a.total_work + 7) / 8;
  a.c = 1.4426950408889634f / sqrtf(float(p.head_dim));
  const dim3 grid((unsigned)(a.work_per_xcd * 8));
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kPairBytes) != hipSuccess)
      return finish_launch("hipFuncSetAttribute");
    attr_set = true;
  }
  hipLaunchKernelGGL(attn_bf16_kernel, grid, dim3(256), 2 * kPairBytes,
                     static_cast<hipStream_t>(stream), a);
  return finish_launch("attn_bf16.hip");
}

}  // namespace ca
