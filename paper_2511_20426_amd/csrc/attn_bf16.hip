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
//   tiles), a workgroup 256 rows of one head.  K and V pages (32 KB each) stream global -> LDS
//   without passing through registers into two 2-page rings shared by the four waves.
//   S^T = K Q^T   : v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q (AGPRs).
//                   In the 32x32 accumulator layout a lane then holds 16 of the 32 keys of ONE
//                   query, so row max / row sum need a single cross-lane step (lane ^ 32), and
//                   only on the rare steps where the exponent reference moves.
//   O^T += V^T P^T: A = V^T rows from LDS, B = P^T straight from the S^T accumulator
//                   registers (rounded to bf16).  V pages are stored transposed and with the
//                   key order the accumulator hands over, so no data movement is needed
//                   between the two products (see cascade_attn.h for the page format).
//   Softmax is the running-reference form in base 2: p = exp2(s*c - m_ref), c = log2(e)/sqrt(D);
//   m_ref moves (and the accumulators are rescaled) only when the probabilities of a step sum past 2^16.
//   The 256-byte page rows are stored with their 16-byte chunks XOR-swizzled by (row & 15),
//   which makes every ds_read_b128 of an MFMA operand bank-conflict free.
//   Workgroups are numbered so that the eight XCDs each take a contiguous range of
//   (head, row tile) work: workgroups running together on an XCD stream the same head's pages
//   and share them in that XCD's L2.
//   This file holds the set-up and the epilogue; the software-pipelined main loop is the
//   hand-scheduled assembly emitted by gen_attn_core.py.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>

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

// Rotary embedding of the queries inside the kernel's Q load.  Angles are formed in revolutions:
// pair j turns by pos * freq[j] / 2pi; that factor is split into a 12-bit head and a tail so that
// pos * head is exact in fp32 for pos < 4096 and only its fractional part meets the hardware
// sin / cos (measured: cos and sin within 4.2e-7 of fp64 for every pos < 4096 and every pair).
struct QRope {
  float rev_hi[kMaxPairs], rev_lo[kMaxPairs];
  int32_t pairs_t, pairs_h;            // pairs [0, pairs_t): frame axis, then pairs_h: row axis, rest: column axis
  int32_t grid_w, plane, block_tokens; // plane = grid_h * grid_w
  int32_t first_frame[kMaxInflight];   // of the launch's query blocks
  int64_t tok_stride, head_stride;     // of q, in elements
};

struct AttnArgs {
  const uint16_t* q;
  uint16_t* o;
  const uint8_t* pool;
  int32_t heads, pages_per_block, last_valid;
  // Query segments: rows that share one visible prefix (one segment in a bidirectional cascade,
  // one per query block in a block-causal one, longest prefix first); all have tiles_per_seg row
  // tiles.  A "column" is a (head, row tile) pair; XCD x owns columns [x*cols_per_xcd,
  // (x+1)*cols_per_xcd) and works through them segment by segment: item i of an XCD is segment
  // i / cols_per_xcd of column i % cols_per_xcd.  Workgroups that run together on an XCD then
  // walk KV prefixes of one length, start and finish together, and stay in step on the same pages
  // of the same few heads, which is what keeps those pages in the XCD's L2.
  int32_t n_seg, tiles_per_seg, total_cols, cols_per_xcd;
  int32_t seg_row0[kMaxSeg], seg_rows[kMaxSeg], seg_nvis[kMaxSeg];
  int32_t kv_slot[kMaxKvBlocks];
  int32_t work_per_xcd;                // = cols_per_xcd * n_seg
  // Tail balancing: the last `split_items` work items of every XCD's range have their KV walk cut
  // into `split` page ranges, one workgroup each, so that the launch's last, partly filled round
  // of workgroups is shorter; their partial results meet in merge_partials_kernel.
  int32_t split, split_items, full_items;   // per XCD: full_items + split_items == work_per_xcd
  float* partials;                     // [xcd][split item][chunk][kPartialFloats]
  float c;                             // log2(e) / sqrt(head_dim)
  // Only read by the instantiation that rotates Q itself (attn_bf16_kernel<true>): q is then the
  // unrotated [row, head, dim] tensor with the caller's strides.
  QRope rq;
};

// one partial result of a 256-row tile: O^T contributions [row][128] (fp32, not normalised),
// then the row's exponent reference (log2 units) and row sum
constexpr int kPartialRow = 132;                 // floats per row: 128 + reference + sum, padded to 16 B
constexpr int kPartialFloats = kRowsPerWg * kPartialRow;
static_assert(size_t(kMaxPartials) * kPartialFloats * 4 == kAttnScratchBytes, "scratch size");

struct WorkItem {
  int h, row0, rows_end, n_kvb;     // h < 0: no such item (the last XCD may own fewer columns)
};

__device__ __forceinline__ WorkItem decode_item(const AttnArgs& a, int xcd, int item) {
  WorkItem w;
  const int seg = item / a.cols_per_xcd;
  const int col = xcd * a.cols_per_xcd + (item - seg * a.cols_per_xcd);
  if (seg >= a.n_seg || col >= a.total_cols) {
    w.h = -1;
    w.row0 = w.rows_end = w.n_kvb = 0;
    return w;
  }
  w.h = col / a.tiles_per_seg;
  const int t = col - w.h * a.tiles_per_seg;
  w.row0 = a.seg_row0[seg] + t * kRowsPerWg;
  w.rows_end = a.seg_row0[seg] + a.seg_rows[seg];
  w.n_kvb = a.seg_nvis[seg];
  return w;
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);   // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(uint32_t, b);
}

// value of the partner lane (lane ^ 32)
__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }

#include "attn_core_clobbers.inc"

// LDS map: K ring (2 pages) then V ring (2 pages); the main loop lives in attn_core_gfx950.inc
// (generated by gen_attn_core.py, which also documents the pipeline and the register map).
constexpr uint32_t kVRing = 2 * kPageBytes;

template <bool kRopeQ>
__global__ __launch_bounds__(256, 1) void attn_bf16_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, hi = lane >> 5, sw = lane & 15;

  // ---- which (head, row tile, page range): XCD x takes its own work_per_xcd items;
  // inside an XCD the full items come first, then `split` workgroups per split item
  const int xcd = blockIdx.x & 7, nth = blockIdx.x >> 3;
  int item = nth, chunk = 0, n_chunks = 1;
  if (nth >= a.full_items) {
    item = a.full_items + (nth - a.full_items) / a.split;
    chunk = (nth - a.full_items) % a.split;
    n_chunks = a.split;
  }
  if (item >= a.work_per_xcd) return;
  const WorkItem wi = decode_item(a, xcd, item);
  if (wi.h < 0) return;
  const int h = wi.h, row0 = wi.row0, rows_end = wi.rows_end, n_kvb = wi.n_kvb;
  const int all_pages = n_kvb * a.pages_per_block;
  const int page_lo = int(int64_t(all_pages) * chunk / n_chunks);
  const int page_hi = int(int64_t(all_pages) * (chunk + 1) / n_chunks);
  const int n_pages = page_hi - page_lo;
  const int kb0 = page_lo / a.pages_per_block, pg0 = page_lo - kb0 * a.pages_per_block;

  // ---- Q fragments: B operand of S^T = K Q^T.  Lane holds dims 16ks + 8hi .. +7 of query l31
  // of column tile nt; fragment (nt, ks) goes to a[128 + 4*(8nt + ks) ..].
  // The instantiation that rotates Q itself does so in a pass of its own: thread t rotates row t of
  // the workgroup's 256 rows, scales, rounds once and parks the row in LDS, which the page rings do
  // not use yet; the fragment loads below then read LDS.
  if (kRopeQ) {
    const int r = row0 + tid;
    const bool ok = r < rows_end;
    const int rr = ok ? r : row0;
    const int blk = rr / a.rq.block_tokens, n = rr - blk * a.rq.block_tokens;
    const int fr = n / a.rq.plane, in_plane = n - fr * a.rq.plane;
    const int y = in_plane / a.rq.grid_w;
    const float pos_f = float(a.rq.first_frame[blk] + fr), pos_y = float(y), pos_x = float(in_plane - y * a.rq.grid_w);
    const uint16_t* qp = a.q + int64_t(rr) * a.rq.tok_stride + int64_t(h) * a.rq.head_stride;
    u32x4 v[16];                                            // the row's 16 chunks, all loads in flight at once
#pragma unroll
    for (int c = 0; c < 16; ++c) v[c] = *reinterpret_cast<const u32x4*>(qp + 8 * c);
    // the per-pair factors go through LDS (behind the 64 KB the rotated rows will take): read from
    // the argument block with compile-time indices they would sit in 128 scalar registers
    float* tab = reinterpret_cast<float*>(lds + 65536);
    if (tid < 2 * kMaxPairs) tab[tid] = tid < kMaxPairs ? a.rq.rev_hi[tid] : a.rq.rev_lo[tid - kMaxPairs];
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 16; ++c) {                          // chunk c: dims 8c .. 8c+7, pairs 4c .. 4c+3
      u32x4 out;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int pair = 4 * c + j;
        const float pos = pair < a.rq.pairs_t ? pos_f : (pair < a.rq.pairs_t + a.rq.pairs_h ? pos_y : pos_x);
        const float rev = __builtin_amdgcn_fractf(pos * tab[pair]) + pos * tab[kMaxPairs + pair];
        const float cs = __builtin_amdgcn_cosf(rev), sn = __builtin_amdgcn_sinf(rev);
        const uint32_t x = ok ? v[c][j] : 0u;
        const float u = __uint_as_float(x << 16), w = __uint_as_float(x & 0xffff0000u);
        // scores come out of the matrix pipe in log2 units: Q is scaled by c = log2(e)/sqrt(D) here
        out[j] = pack2((u * cs - w * sn) * a.c, (u * sn + w * cs) * a.c);
      }
      *reinterpret_cast<u32x4*>(lds + tid * 256 + ((c ^ (tid & 15)) << 4)) = out;
    }
    __syncthreads();
  }
  int qrow[2];
  f32x16 qt[4];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int lrow = wave * 64 + nt * 32 + l31;              // row inside the workgroup's tile
    qrow[nt] = row0 + lrow;
    const bool ok = qrow[nt] < rows_end;
    const uint16_t* qp = a.q + (int64_t(ok ? qrow[nt] : row0) * a.heads + h) * 128 + hi * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      if (kRopeQ) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(lds + lrow * 256 + (((2 * ks + hi) ^ (lrow & 15)) << 4));
#pragma unroll
        for (int j = 0; j < 4; ++j) qt[2 * nt + (ks >> 2)][4 * (ks & 3) + j] = __uint_as_float(v[j]);
      } else {
        u32x4 v = *reinterpret_cast<const u32x4*>(qp + ks * 16);
        if (!ok) v = u32x4{0, 0, 0, 0};
        // scores come out of the matrix pipe in log2 units: Q is scaled by c = log2(e)/sqrt(D) here
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t w = pack2(__uint_as_float(v[j] << 16) * a.c, __uint_as_float(v[j] & 0xffff0000u) * a.c);
          qt[2 * nt + (ks >> 2)][4 * (ks & 3) + j] = __uint_as_float(w);
        }
      }
    }
  }
  if (kRopeQ) __syncthreads();        // every fragment is in registers before the first page lands in LDS

  // address of page 0 of KV block i for this head: lane i of (tbl_lo, tbl_hi)
  const int my_slot = a.kv_slot[lane & (kMaxKvBlocks - 1)];
  const uint64_t my_off = reinterpret_cast<uint64_t>(a.pool) +
                          (uint64_t(my_slot) * a.pages_per_block * a.heads + h) * uint64_t(kPairBytes);
  const uint32_t tbl_lo = uint32_t(my_off), tbl_hi = uint32_t(my_off >> 32);
  const uint32_t xo0 = l31 * 256 + ((hi ^ sw) << 4);    // row offset + swizzled chunk 0 (or 1 for hi)
  const uint32_t lane_off = wave * 1024 + lane * 16;   // this lane's 16 bytes inside each 4 KB slice of a page
  const uint32_t kidx = 4 * hi;
  const uint32_t xlane = 4 * (lane ^ 32);
  const uint32_t stride = uint32_t(a.heads) * kPairBytes;
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);

  // The first PV product multiplies an all-zero P tile with whatever the second V ring slot
  // holds: make that finite.
#pragma unroll
  for (int i = 0; i < 8; ++i)
    *reinterpret_cast<u32x4*>(lds + kVRing + kPageBytes + (i * 256 + tid) * 16) = u32x4{0, 0, 0, 0};

  // o6/o7 are not early-clobber: the block reads every VGPR input in its first instructions,
  // before it writes v[96:127], and the inputs need somewhere to live (it uses all of v[128:255])
  f32x16 o0, o1, o2, o3, o4, o5, o6, o7;
  float l0a, l0b, l1a, l1b, negm0, negm1;
  asm volatile(
#include "attn_core_gfx950.inc"
      : "=&{v[0:15]}"(o0), "=&{v[16:31]}"(o1), "=&{v[32:47]}"(o2), "=&{v[48:63]}"(o3), "=&{v[64:79]}"(o4),
        "=&{v[80:95]}"(o5), "={v[96:111]}"(o6), "={v[112:127]}"(o7), "=&{v148}"(l0a), "=&{v149}"(l0b),
        "=&{v150}"(l1a), "=&{v151}"(l1b), "=&{v184}"(negm0), "=&{v200}"(negm1)
      : "{a[128:143]}"(qt[0]), "{a[144:159]}"(qt[1]), "{a[160:175]}"(qt[2]), "{a[176:191]}"(qt[3]),
        [xo0] "v"(xo0), [lane_off] "v"(lane_off), [tbl_lo] "v"(tbl_lo), [tbl_hi] "v"(tbl_hi),
        [kidx] "v"(kidx), [xlane] "v"(xlane), [n_pages] "s"(n_pages), [n_kvb] "s"(n_kvb), [kb0] "s"(kb0), [pg0] "s"(pg0),
        [ppb] "s"(a.pages_per_block), [stride] "s"(stride), [last_valid] "s"(a.last_valid),
        [wave] "s"(wave_s), [lds0] "s"(lds0)
      : "memory", "vcc", "scc", "m0", CA_CORE_CLOBBERS);

  // ---- normalise and store: lane holds, for its query, dims 32mt + 8(i/4) + 4hi + (i%4)
  const f32x16 oacc[4][2] = {{o0, o1}, {o2, o3}, {o4, o5}, {o6, o7}};
  const float l_lane[2] = {l0a + l0b, l1a + l1b};
  if (n_chunks > 1) {
    // partial result: accumulators as they are, plus (m_ref, row sum) per row
    float* part = a.partials + (size_t(xcd * a.split_items + (item - a.full_items)) * a.split + chunk) * kPartialFloats;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const float l_tot = l_lane[nt] + other_half(l_lane[nt]);
      const int r = wave * 64 + nt * 32 + l31;
      float* rp = part + r * kPartialRow;
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x16& o = oacc[mt][nt];
          const float x0 = o[4 * g + 0], x1 = o[4 * g + 1], x2 = o[4 * g + 2], x3 = o[4 * g + 3];
          *reinterpret_cast<float4*>(rp + 32 * mt + 8 * g + 4 * hi) = make_float4(x0, x1, x2, x3);
        }
      if (hi == 0) {
        rp[128] = -(nt ? negm1 : negm0);
        rp[129] = l_tot;
      }
    }
    return;
  }
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float l_tot = l_lane[nt] + other_half(l_lane[nt]);
    const float inv = 1.0f / l_tot;
    if (qrow[nt] < rows_end) {
      uint16_t* op = a.o + (int64_t(qrow[nt]) * a.heads + h) * 128 + 4 * hi;
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x16& o = oacc[mt][nt];
          u32x2 w;
          w[0] = pack2(o[4 * g + 0] * inv, o[4 * g + 1] * inv);
          w[1] = pack2(o[4 * g + 2] * inv, o[4 * g + 3] * inv);
          *reinterpret_cast<u32x2*>(op + 32 * mt + 8 * g) = w;
        }
    }
  }
}


// Combines the partial results of the split work items: for every row, the partials are brought
// to the largest of their exponent references, summed and normalised.  Eight workgroups per tile
// (blockIdx.y picks 32 of its rows); 32 threads share a row (four dims each), so that a row of a
// partial tile is read as 512 contiguous bytes and a result row is written as 256.
__global__ __launch_bounds__(256) void merge_partials_kernel(AttnArgs a) {
  const int xcd = blockIdx.x / a.split_items, sidx = blockIdx.x % a.split_items;
  const WorkItem wi = decode_item(a, xcd, a.full_items + sidx);
  if (wi.h < 0) return;
  const int sub = threadIdx.x >> 5, d = 4 * (threadIdx.x & 31);
  const float* tile = a.partials + size_t(xcd * a.split_items + sidx) * a.split * kPartialFloats;
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int r = int(blockIdx.y) * 32 + pass * 8 + sub;
    const int row = wi.row0 + r;
    if (row >= wi.rows_end) break;                       // rows only grow from here
    const float* part = tile + r * kPartialRow;
    float m = -INFINITY;
    for (int c = 0; c < a.split; ++c) m = fmaxf(m, part[c * kPartialFloats + 128]);
    float l = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int c = 0; c < a.split; ++c) {
      const float wgt = __builtin_amdgcn_exp2f(part[c * kPartialFloats + 128] - m);
      l += wgt * part[c * kPartialFloats + 129];
      const float4 x = *reinterpret_cast<const float4*>(part + c * kPartialFloats + d);
      acc.x += wgt * x.x; acc.y += wgt * x.y; acc.z += wgt * x.z; acc.w += wgt * x.w;
    }
    const float inv = 1.0f / l;
    u32x2 w;
    w[0] = pack2(acc.x * inv, acc.y * inv);
    w[1] = pack2(acc.z * inv, acc.w * inv);
    *reinterpret_cast<u32x2*>(a.o + (int64_t(row) * a.heads + wi.h) * 128 + d) = w;
  }
}

}  // namespace

// variant 0: default; 1: no tail balancing (every work item walks its whole KV range)
int32_t attn_bf16_variant_ok(int variant) { return variant == 0 || variant == 1 ? CA_OK : CA_EINVAL; }

namespace {

// Fills the kernel arguments for one forward.  Tail balancing: `capacity` partial results fit in
// the scratch area; with adapt the split is reduced until the partials fit, without it the split
// the device's CU count asks for is kept and *partials_needed tells the caller how many it takes.
int32_t plan_attn_bf16(const AttnPlan& p, int variant, const void* q, void* out, const void* pool, void* partials_dev,
                       int capacity, bool adapt, AttnArgs* args, int* partials_needed) {
  if (p.head_dim != 128 || p.page_tokens != 128) return CA_EUNSUPPORTED;
  if (attn_bf16_variant_ok(variant) != CA_OK) return CA_EINVAL;
  AttnArgs& a = *args;
  a = AttnArgs{};
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
    tiles = (a.seg_rows[0] + kRowsPerWg - 1) / kRowsPerWg;
  } else {
    // one segment per query block, the longest prefix (latest block) first
    a.n_seg = p.n_q_blocks;
    for (int j = 0; j < p.n_q_blocks; ++j) {
      const int i = p.n_q_blocks - 1 - j;
      a.seg_row0[j] = i * p.block_tokens;
      a.seg_rows[j] = p.block_tokens;
      a.seg_nvis[j] = p.n_vis[i];
    }
    tiles = (p.block_tokens + kRowsPerWg - 1) / kRowsPerWg;
  }
  a.tiles_per_seg = tiles;
  a.total_cols = tiles * p.heads;
  a.cols_per_xcd = (a.total_cols + 7) / 8;
  a.work_per_xcd = a.cols_per_xcd * a.n_seg;
  a.c = 1.4426950408889634f / sqrtf(float(p.head_dim));
  // Tail balancing.  One workgroup occupies a CU, an XCD has n_cu/8 of them, and all items of a
  // launch take about the same time: after floor(items / cus) full rounds, `rem` items would run
  // alone while the other CUs idle.  Their KV walks are cut into split = floor(cus / rem) ranges.
  int n_cu = 0;
  if (const int32_t rc = device_cu_count(&n_cu); rc != CA_OK) return rc;
  const int cus_per_xcd = n_cu >= 8 ? n_cu / 8 : 1;
  a.split = 1;
  a.split_items = 0;
  a.full_items = a.work_per_xcd;
  a.partials = static_cast<float*>(partials_dev);
  const int rem = a.work_per_xcd % cus_per_xcd;
  int min_vis = p.n_vis[0];                                    // shortest KV walk of the launch
  for (int i = 1; i < p.n_q_blocks; ++i) min_vis = p.n_vis[i] < min_vis ? p.n_vis[i] : min_vis;
  const int min_pages = min_vis * p.pages_per_block;
  *partials_needed = 0;
  if (partials_dev && variant == 0 && rem > 0 && a.work_per_xcd > cus_per_xcd) {
    int split = cus_per_xcd / rem;
    if (split > 8) split = 8;
    while (split > 1 && (min_pages < 8 * split || (adapt && 8 * rem * split > capacity))) --split;
    if (split > 1) {
      a.split = split;
      a.split_items = rem;
      a.full_items = a.work_per_xcd - rem;
      *partials_needed = 8 * rem * split;
    }
  }
  return CA_OK;
}

int32_t enqueue_attn_bf16(const AttnArgs& a, bool rope_q, void* stream) {
  const dim3 grid((unsigned)((a.full_items + a.split_items * a.split) * 8));
  const void* kernel = rope_q ? reinterpret_cast<const void*>(attn_bf16_kernel<true>)
                              : reinterpret_cast<const void*>(attn_bf16_kernel<false>);
  if (const int32_t rc = ensure_dynamic_lds(kernel, 4 * kPageBytes, rope_q ? 2 : 0); rc != CA_OK) return rc;
  if (rope_q)
    hipLaunchKernelGGL(attn_bf16_kernel<true>, grid, dim3(256), 4 * kPageBytes, static_cast<hipStream_t>(stream), a);
  else
    hipLaunchKernelGGL(attn_bf16_kernel<false>, grid, dim3(256), 4 * kPageBytes, static_cast<hipStream_t>(stream), a);
  if (a.split > 1)
    hipLaunchKernelGGL(merge_partials_kernel, dim3((unsigned)(8 * a.split_items), kRowsPerWg / 32), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
  return finish_launch("attn_bf16.hip");
}

}  // namespace

int32_t launch_attn_bf16(const AttnPlan& p, int variant, const void* q, void* out, const void* pool,
                         void* partials_dev, int max_partials, void* stream) {
  AttnArgs a;
  int needed = 0;
  if (const int32_t rc = plan_attn_bf16(p, variant, q, out, pool, partials_dev, max_partials, true, &a, &needed);
      rc != CA_OK)
    return rc;
  return enqueue_attn_bf16(a, false, stream);
}

int32_t launch_attn_bf16_rope(const AttnPlan& p, const QRopePlan& rp, int variant, const void* q, void* out,
                              const void* pool, void* partials_dev, int max_partials, void* stream) {
  AttnArgs a;
  int needed = 0;
  if (const int32_t rc = plan_attn_bf16(p, variant, q, out, pool, partials_dev, max_partials, true, &a, &needed);
      rc != CA_OK)
    return rc;
  const double two_pi = 6.283185307179586476925286766559;
  for (int j = 0; j < kMaxPairs; ++j) {
    const double rev = rp.geom.freq[j] / two_pi;
    int e = 0;
    const double m = std::frexp(rev, &e);                       // rev = m 2^e, 0.5 <= m < 1
    const double head = std::ldexp(std::floor(std::ldexp(m, 12)), e - 12);
    a.rq.rev_hi[j] = float(head);
    a.rq.rev_lo[j] = float(rev - head);
  }
  a.rq.pairs_t = rp.geom.pairs_t;
  a.rq.pairs_h = rp.geom.pairs_h;
  a.rq.grid_w = rp.geom.grid_w;
  a.rq.plane = rp.geom.grid_h * rp.geom.grid_w;
  a.rq.block_tokens = p.block_tokens;
  for (int i = 0; i < p.n_q_blocks; ++i) {
    // positions must stay below 4096 for the exact head product (frames are the only axis that grows)
    if (rp.first_frame[i] < 0 || rp.first_frame[i] + p.block_tokens / a.rq.plane >= 4096) return CA_EUNSUPPORTED;
    a.rq.first_frame[i] = int32_t(rp.first_frame[i]);
  }
  if (rp.geom.grid_h >= 4096 || rp.geom.grid_w >= 4096) return CA_EUNSUPPORTED;
  a.rq.tok_stride = rp.tok_stride;
  a.rq.head_stride = rp.head_stride;
  return enqueue_attn_bf16(a, true, stream);
}

// ---- the same launch with the partial results in device memory this library holds itself, for
// callers that cannot hand over or allocate any: a file-scope array, one copy per GPU, which
// stays with the process.  Host code never uses the array's name as an address: the address on
// the current device is looked up once per device and kept.
namespace {

constexpr int kStaticPartials = 256;      // 256 tiles x 256 rows x 132 floats = 34.6 MB per GPU
static __device__ __align__(256) float scratch[size_t(kStaticPartials) * kPartialFloats];

std::atomic<float*> g_static_scratch[kMaxDevices];

int32_t static_scratch_on_current_device(float** out) {
  int dev = 0;
  if (const hipError_t e = hipGetDevice(&dev); e != hipSuccess) return device_failure("hipGetDevice", e);
  if (dev < 0 || dev >= kMaxDevices) return CA_EUNSUPPORTED;
  float* ptr = g_static_scratch[dev].load(std::memory_order_acquire);
  if (!ptr) {
    void* sym = nullptr;
    if (const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)); e != hipSuccess || !sym)
      return device_failure("hipGetSymbolAddress(scratch)", e);
    ptr = static_cast<float*>(sym);
    g_static_scratch[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return CA_OK;
}

}  // namespace

void attn_static_scratch_prepare() {
  float* ptr = nullptr;
  if (static_scratch_on_current_device(&ptr) != CA_OK) (void)hipGetLastError();   // the entry point will try again
}

int32_t launch_attn_bf16_static(const AttnPlan& p, int variant, const void* q, void* out, const void* pool,
                                void* stream) {
  float* ptr = nullptr;
  if (const int32_t rc = static_scratch_on_current_device(&ptr); rc != CA_OK) return rc;
  AttnArgs a;
  int needed = 0;
  // the split the device's CU count asks for, as launch_attn_bf16 takes it when its area is large
  // enough; what does not fit the static area is refused, not shrunk
  if (const int32_t rc = plan_attn_bf16(p, variant, q, out, pool, ptr, kStaticPartials, false, &a, &needed); rc != CA_OK)
    return rc;
  if (needed > kStaticPartials) return CA_ETOOBIG;
  return enqueue_attn_bf16(a, false, stream);
}

}  // namespace ca
