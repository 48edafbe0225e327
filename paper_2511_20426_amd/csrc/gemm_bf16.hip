// Y[M,N] = X[M,K] . W[N,K]^T in bf16 with fp32 accumulation: the linear maps either side of the
// attention inside a DiT layer (QKV projection before it, output projection after it).
//
//   Workgroup = 4 waves = a 256 x 256 tile of Y, one wave per SIMD; the main loop (K in stages of
//   64, both operands through rings in LDS that together fill its 160 KB) is the assembly
//   emitted by gen_gemm_core.py, which documents the pipeline and the register map.  This file
//   holds the set-up, the epilogue (tile transposed through LDS so that rows of Y are written as
//   256-byte runs) and the launch.
//   Workgroups are numbered so that the 32 running together on one XCD form an 8 x 4 block of
//   tiles: they share 8 row slabs of X and 4 row slabs of W in that XCD's L2.
//
//   A second instantiation is the QKV projection of the blocks in flight with the publication of
//   their K/V fused into its epilogue (Sec. 3.3: every block's K/V go to the shared pool at every
//   self-attention layer): row tiles are counted per block, so that a wave's 128 x 128 sub-tile is
//   exactly one page of one head; K sub-tiles are rotated and stored as K pages, V sub-tiles are
//   stored transposed as V pages, Q sub-tiles go to a packed tensor -- the same bytes the separate
//   cache-write kernel produces from the projection's output, without that output ever being
//   written.
#include <hip/hip_runtime.h>

#include "ca_internal.hpp"

namespace ca {
namespace {

#include "rope_device.hpp"

typedef __attribute__((ext_vector_type(16))) uint32_t u32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kTile = 256;
constexpr int kSbRows = 8, kSbCols = 4;           // tiles of one XCD's block
constexpr int kEpiRow = 272;                      // bytes per row of a wave's 128 x 128 bf16 tile in LDS
constexpr int kEpiRowV = 260;                     // the same for a V sub-tile of the publishing epilogue, which is read
                                                  // back two bytes at a time down its columns: 65 dwords per row spread
                                                  // the 16 token groups a wave reads at once over 16 banks
constexpr int kEpiWave = 128 * kEpiRow;
constexpr int kGemmLds = 160 * 1024;              // main loop: 3 W stages + 2 X stages of 32 KB; epilogue: 4 x kEpiWave
static_assert(4 * kEpiWave + 2 * 12288 <= kGemmLds, "epilogue staging and two trig tables fit");

// What the publishing epilogue needs beyond the product itself.
struct PublishArgs {
  RopeGeom g;
  uint8_t* pool;
  int32_t heads, pages_per_block;
  int32_t slot[kMaxInflight];
  int64_t first_frame[kMaxInflight];
  TrigTable tab;                                  // per-page cos/sin table (n_f == 0: threads evaluate their own)
};

struct GemmArgs {
  const uint16_t* x;
  const uint16_t* w;
  uint16_t* y;                                    // publishing: the packed queries [M][heads * 128]
  int32_t M, N, K;
  int64_t ldx, ldw, ldy;                          // row strides in elements
  int32_t tiles_m, tiles_n, sb_cols, n_sb;
  // Row tiles are counted inside row blocks of block_rows rows, tiles_per_block each (the last
  // one ragged): one block spanning all of M for the plain product, one per in-flight block when
  // publishing.
  int32_t block_rows, tiles_per_block;
  PublishArgs pub;                                // read by gemm_bf16_kernel<true> only
};

constexpr int kTrigBytes = 12288;                 // per 128-token page; two pages per workgroup behind the staging area

#include "gemm_core_clobbers.inc"

template <bool kPublish>
__global__ __launch_bounds__(256, 1) void gemm_bf16_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, grp = lane >> 4;
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  const int sb = (j >> 5) * 8 + xcd, within = j & 31;
  if (sb >= a.n_sb) return;
  const int tm = (sb / a.sb_cols) * kSbRows + (within & 7);
  const int tn = (sb % a.sb_cols) * kSbCols + (within >> 3);
  if (tm >= a.tiles_m || tn >= a.tiles_n) return;
  const int blk = tm / a.tiles_per_block, tile_in_blk = tm - blk * a.tiles_per_block;
  const int m0 = blk * a.block_rows + tile_in_blk * kTile, n0 = tn * kTile;
  const int m_end = min((blk + 1) * a.block_rows, a.M);           // first row past this tile's row block
  const int wm = wave & 1, wn = wave >> 1;

  // load i of this wave brings rows (8 wave + i) 8 .. +7 of a part (128-byte rows: whole cache
  // lines); lane L brings what is stored at position L & 7 of row L >> 3: chunk (L & 7) ^ ((row >> 1) & 7)
  uint32_t offw[8], offx[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = (wave * 8 + i) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    const int nrow = min(n0 + row, a.N - 1) - n0;                // rows of w past n_out re-read its last row
    offw[i] = uint32_t(int64_t(nrow) * a.ldw * 2 + c * 16);
    const int mrow = min(m0 + row, m_end - 1) - m0;              // rows past the block's end re-read its last row
    offx[i] = uint32_t(int64_t(mrow) * a.ldx * 2 + c * 16);
  }
  const uint64_t base_w = reinterpret_cast<uint64_t>(a.w + int64_t(n0) * a.ldw);
  const uint64_t base_x = reinterpret_cast<uint64_t>(a.x + int64_t(m0) * a.ldx);
  // operand reads (16 x 16 x 32 MFMA: lane = row l15 of a 16-row sub-tile, 8 k-values of group
  // grp): chunk grp of k-step 0 of the lane's row in the wave's 128 rows
  const uint32_t swz = (l15 >> 1) & 7;
  const uint32_t aw0 = uint32_t((wn * 128 + l15) * 128) + ((uint32_t(grp) ^ swz) << 4);
  const uint32_t ax0 = uint32_t((wm * 128 + l15) * 128) + ((uint32_t(grp) ^ swz) << 4);
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int n_stages = a.K / 64;

  u32x16 o0, o1, o2, o3, o4, o5, o6, o7;
  asm volatile(
#include "gemm_core_gfx950.inc"
      : "=&{v[0:15]}"(o0), "=&{v[16:31]}"(o1), "=&{v[32:47]}"(o2), "=&{v[48:63]}"(o3), "=&{v[64:79]}"(o4),
        "=&{v[80:95]}"(o5), "=&{v[96:111]}"(o6), "=&{v[112:127]}"(o7)
      : [base_w] "s"(base_w), [base_x] "s"(base_x), [n_stages] "s"(n_stages), [wave] "s"(wave_s),
        [lds0] "s"(lds0), [offw0] "v"(offw[0]), [offw1] "v"(offw[1]), [offw2] "v"(offw[2]), [offw3] "v"(offw[3]),
        [offw4] "v"(offw[4]), [offw5] "v"(offw[5]), [offw6] "v"(offw[6]), [offw7] "v"(offw[7]),
        [offx0] "v"(offx[0]), [offx1] "v"(offx[1]), [offx2] "v"(offx[2]), [offx3] "v"(offx[3]),
        [offx4] "v"(offx[4]), [offx5] "v"(offx[5]), [offx6] "v"(offx[6]), [offx7] "v"(offx[7]),
        [aw0] "v"(aw0), [ax0] "v"(ax0)
      : "memory", "scc", "m0", CA_GEMM_CLOBBERS);

  // ---- epilogue: the wave's 128 (m) x 128 (n) tile goes through LDS to come out row by row.
  // Pair p of MFMA tile T = 8 ti + tj: n = 16 ti + 4 grp + 2 p, m = 16 tj + l15.
  __syncthreads();                                    // every wave is done with the stage buffers
  uint8_t* mine = lds + wave * kEpiWave;
  const int v_section = kPublish && (n0 + wn * 128) / (a.pub.heads * 128) == 2;
  const int pitch = v_section ? kEpiRowV : kEpiRow;
  const u32x16 o[8] = {o0, o1, o2, o3, o4, o5, o6, o7};
#pragma unroll
  for (int T = 0; T < 64; ++T) {
    const int ti = T >> 3, tj = T & 7;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int n = 16 * ti + 4 * grp + 2 * p;
      const int m = 16 * tj + l15;
      *reinterpret_cast<uint32_t*>(mine + m * pitch + n * 2) = o[(2 * T + p) >> 4][(2 * T + p) & 15];
    }
  }
  __syncthreads();
  if (!kPublish) {
#pragma unroll 4
    for (int it = 0; it < 32; ++it) {
      const int row = it * 4 + (lane >> 4), c = lane & 15;
      const u32x4 v = *reinterpret_cast<const u32x4*>(mine + row * kEpiRow + c * 16);
      const int gm = m0 + wm * 128 + row;
      // the result passes through once: keep it from displacing the operand tiles in the caches
      if (gm < m_end && n0 + wn * 128 + c * 8 < a.N)            // n_out is a multiple of 8: a chunk is inside or outside
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(a.y + int64_t(gm) * a.ldy + n0 + wn * 128 + c * 8));
    }
    return;
  }
  // ---- publishing epilogue.  The wave's sub-tile is one head of q, k or v (output rows are
  // ordered q|k|v, head, dim) for the 128 tokens of page 2 * tile_in_blk + wm of block blk.
  const PublishArgs& pb = a.pub;
  const int width = pb.heads * 128;
  const int col = n0 + wn * 128;
  const int section = col / width, head = (col - section * width) >> 7;      // the same for all four waves' section
  const int page = 2 * tile_in_blk + wm;
  const int tok0 = page * 128;                                                // first token of the page in its block
  const int c = lane & 15, r4 = lane >> 4;
  if (section == 0) {                      // q: as it is (the attention kernel rotates it), packed rows
#pragma unroll 4
    for (int it = 0; it < 32; ++it) {
      const int row = it * 4 + r4;
      const u32x4 v = *reinterpret_cast<const u32x4*>(mine + row * kEpiRow + c * 16);
      if (tok0 + row < a.block_rows)
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(a.y + int64_t(m0 + wm * 128 + row) * a.ldy + head * 128 + c * 8));
    }
    return;
  }
  const bool has_page = page < pb.pages_per_block;
  uint8_t* kpage = pb.pool + ((int64_t(pb.slot[blk]) * pb.pages_per_block + (has_page ? page : 0)) * pb.heads + head) *
                                 int64_t(2 * 128 * 128 * 2);
  if (section == 1) {                      // k: rotate by the token's position, K page rows, pad rows zero
    float2* trig = reinterpret_cast<float2*>(lds + 4 * kEpiWave + wm * kTrigBytes);
    TrigLayout lay{};
    if (pb.tab.n_f > 0) {                  // the two waves of a page (wn = 0, 1) fill its table together
      lay = trig_layout(pb.g, pb.tab, tok0, a.block_rows, pb.first_frame[blk]);
      if (has_page) trig_fill(pb.g, lay, trig, wn * 64 + lane, 128);
    }
    __syncthreads();
    if (!has_page) return;
    // the lane's rows are tokens tok0 + r4 + 4 it: positions move on by four tokens per trip
    TokenPos p = token_pos(min(tok0 + r4, a.block_rows - 1), pb.first_frame[blk], pb.g.grid_h, pb.g.grid_w);
#pragma unroll 2
    for (int it = 0; it < 32; ++it, p = token_advance(p, 4, pb.g.grid_h, pb.g.grid_w)) {
      const int row = it * 4 + r4;
      U4 kk = {0, 0, 0, 0};
      if (tok0 + row < a.block_rows) {
        float cs[4], sn[4];
        if (pb.tab.n_f > 0) {
          trig_pick(pb.g, lay, trig, p, c, cs, sn);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) pair_cs<false>(pb.g, p, c * 4 + j, &cs[j], &sn[j]);
        }
        const U4 raw = *reinterpret_cast<const U4*>(mine + row * kEpiRow + c * 16);
        Vec8<uint16_t> e;
        e.v[0] = bf16_lo(raw.x); e.v[1] = bf16_hi(raw.x); e.v[2] = bf16_lo(raw.y); e.v[3] = bf16_hi(raw.y);
        e.v[4] = bf16_lo(raw.z); e.v[5] = bf16_hi(raw.z); e.v[6] = bf16_lo(raw.w); e.v[7] = bf16_hi(raw.w);
        rotate8(e, cs, sn);
        kk.x = pack_bf16(e.v[0], e.v[1]); kk.y = pack_bf16(e.v[2], e.v[3]);
        kk.z = pack_bf16(e.v[4], e.v[5]); kk.w = pack_bf16(e.v[6], e.v[7]);
      }
      store_once(kpage + row * 256 + ((c ^ (row & 15)) << 4), kk);
    }
    return;
  }
  // v: V page rows are dims; chunk c of a row holds tokens 16 (c / 2) + 4 (c % 2) + {0..3, 8..11}
  if (!has_page) return;
  uint8_t* vpage = kpage + 128 * 128 * 2;
  const int tb = 16 * (c >> 1) + 4 * (c & 1);
#pragma unroll 2
  for (int it = 0; it < 32; ++it) {
    const int d = it * 4 + r4;
    uint32_t e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int tok = tb + (j & 3) + 8 * (j >> 2);
      const uint32_t w = *reinterpret_cast<const uint16_t*>(mine + tok * kEpiRowV + d * 2);
      e[j] = tok0 + tok < a.block_rows ? w : 0u;
    }
    U4 o;
    o.x = e[0] | (e[1] << 16); o.y = e[2] | (e[3] << 16);
    o.z = e[4] | (e[5] << 16); o.w = e[6] | (e[7] << 16);
    store_once(vpage + d * 256 + ((c ^ (d & 15)) << 4), o);
  }
}

}  // namespace

namespace {

int32_t check_gemm_shape(int64_t M, int32_t N, int32_t K, int64_t ldx, int64_t ldw, int64_t ldy) {
  if (M < 0) return CA_EINVAL;
  if (M > (int64_t(1) << 30) || N < 8 || N % 8 != 0 || K < 128 || K % 128 != 0) return CA_EUNSUPPORTED;
  if (ldx < K || ldw < K || ldy < 0 || ldx % 8 != 0 || ldw % 8 != 0 || ldy % 8 != 0) return CA_EINVAL;
  if (ldx * 2 * kTile >= (int64_t(1) << 31) || ldw * 2 * kTile >= (int64_t(1) << 31)) return CA_EUNSUPPORTED;
  return CA_OK;
}

template <bool kPublish>
int32_t enqueue_gemm(GemmArgs& a, void* stream) {
  a.tiles_n = (a.N + kTile - 1) / kTile;
  a.sb_cols = (a.tiles_n + kSbCols - 1) / kSbCols;
  a.n_sb = ((a.tiles_m + kSbRows - 1) / kSbRows) * a.sb_cols;
  const unsigned rounds = unsigned((a.n_sb + 7) / 8);
  if (const int32_t rc = ensure_dynamic_lds(reinterpret_cast<const void*>(gemm_bf16_kernel<kPublish>), kGemmLds,
                                            kPublish ? 3 : 1);
      rc != CA_OK)
    return rc;
  hipLaunchKernelGGL(gemm_bf16_kernel<kPublish>, dim3(rounds * 8 * 32), dim3(256), kGemmLds,
                     static_cast<hipStream_t>(stream), a);
  return finish_launch("gemm_bf16.hip");
}

}  // namespace

int32_t launch_gemm_bf16(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
                         int64_t ldx, int64_t ldw, int64_t ldy, void* stream) {
  if (const int32_t rc = check_gemm_shape(M, N, K, ldx, ldw, ldy); rc != CA_OK) return rc;
  if (ldy < N) return CA_EINVAL;
  if (M == 0) return CA_OK;                       // nothing to do
  GemmArgs a{};
  a.x = static_cast<const uint16_t*>(x);
  a.w = static_cast<const uint16_t*>(w);
  a.y = static_cast<uint16_t*>(y);
  a.M = int32_t(M); a.N = N; a.K = K;
  a.ldx = ldx; a.ldw = ldw; a.ldy = ldy;
  a.tiles_m = int32_t((M + kTile - 1) / kTile);
  a.block_rows = a.M;                             // one row block: tiles run through all of M
  a.tiles_per_block = a.tiles_m;
  return enqueue_gemm<false>(a, stream);
}

int32_t launch_gemm_qkv_publish(const RopeGeom& g, int32_t n_blocks, int32_t block_tokens, int32_t pages_per_block,
                                const int32_t* slot, const int64_t* first_frame, const void* x, int64_t ldx,
                                const void* w, int64_t ldw, int32_t K, void* q_out, void* pool, void* stream) {
  if (g.head_dim != 128 || n_blocks < 1 || n_blocks > kMaxInflight) return CA_EUNSUPPORTED;
  const int32_t N = 3 * g.heads * 128;
  const int64_t M = int64_t(n_blocks) * block_tokens;
  // a 256-wide column tile must not straddle q|k|v: heads * 128 a multiple of 256
  if (g.heads % 2 != 0) return CA_EUNSUPPORTED;
  if (const int32_t rc = check_gemm_shape(M, N, K, ldx, ldw, int64_t(g.heads) * 128); rc != CA_OK) return rc;
  GemmArgs a{};
  a.x = static_cast<const uint16_t*>(x);
  a.w = static_cast<const uint16_t*>(w);
  a.y = static_cast<uint16_t*>(q_out);
  a.M = int32_t(M); a.N = N; a.K = K;
  a.ldx = ldx; a.ldw = ldw; a.ldy = int64_t(g.heads) * 128;
  a.block_rows = block_tokens;
  a.tiles_per_block = (block_tokens + kTile - 1) / kTile;
  a.tiles_m = n_blocks * a.tiles_per_block;
  a.pub.g = g;
  a.pub.pool = static_cast<uint8_t*>(pool);
  a.pub.heads = g.heads;
  a.pub.pages_per_block = pages_per_block;
  for (int i = 0; i < n_blocks; ++i) {
    a.pub.slot[i] = slot[i];
    a.pub.first_frame[i] = first_frame[i];
  }
  size_t tab_bytes = 0;
  a.pub.tab = trig_table_for(g, 128, kTrigBytes, &tab_bytes);
  return enqueue_gemm<true>(a, stream);
}

}  // namespace ca
