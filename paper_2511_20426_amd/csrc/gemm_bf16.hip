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
#include <hip/hip_runtime.h>

#include "ca_internal.hpp"

namespace ca {
namespace {

typedef __attribute__((ext_vector_type(16))) uint32_t u32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kTile = 256;
constexpr int kSbRows = 8, kSbCols = 4;           // tiles of one XCD's block
constexpr int kEpiRow = 272;                      // bytes per row of a wave's 128 x 128 bf16 tile in LDS
constexpr int kEpiWave = 128 * kEpiRow;
constexpr int kGemmLds = 160 * 1024;              // main loop: 3 W stages + 2 X stages of 32 KB; epilogue: 4 x kEpiWave
static_assert(4 * kEpiWave <= kGemmLds, "epilogue staging fits");

struct GemmArgs {
  const uint16_t* x;
  const uint16_t* w;
  uint16_t* y;
  int32_t M, N, K;
  int64_t ldx, ldw, ldy;                          // row strides in elements
  int32_t tiles_m, tiles_n, sb_cols, n_sb;
};

#include "gemm_core_clobbers.inc"

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
  const int m0 = tm * kTile, n0 = tn * kTile;
  const int wm = wave & 1, wn = wave >> 1;

  // load i of this wave brings rows (8 wave + i) 8 .. +7 of a part (128-byte rows: whole cache
  // lines); lane L brings what is stored at position L & 7 of row L >> 3: chunk (L & 7) ^ ((row >> 1) & 7)
  uint32_t offw[8], offx[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = (wave * 8 + i) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    offw[i] = uint32_t(int64_t(row) * a.ldw * 2 + c * 16);
    const int mrow = min(m0 + row, a.M - 1) - m0;                // rows past M re-read the last row
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
  const u32x16 o[8] = {o0, o1, o2, o3, o4, o5, o6, o7};
#pragma unroll
  for (int T = 0; T < 64; ++T) {
    const int ti = T >> 3, tj = T & 7;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int n = 16 * ti + 4 * grp + 2 * p;
      const int m = 16 * tj + l15;
      *reinterpret_cast<uint32_t*>(mine + m * kEpiRow + n * 2) = o[(2 * T + p) >> 4][(2 * T + p) & 15];
    }
  }
  __syncthreads();
#pragma unroll 4
  for (int it = 0; it < 32; ++it) {
    const int row = it * 4 + (lane >> 4), c = lane & 15;
    const u32x4 v = *reinterpret_cast<const u32x4*>(mine + row * kEpiRow + c * 16);
    const int gm = m0 + wm * 128 + row;
    // the result passes through once: keep it from displacing the operand tiles in the caches
    if (gm < a.M)
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(a.y + int64_t(gm) * a.ldy + n0 + wn * 128 + c * 8));
  }
}

}  // namespace

int32_t launch_gemm_bf16(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
                         int64_t ldx, int64_t ldw, int64_t ldy, void* stream) {
  if (M < 0) return CA_EINVAL;
  if (M > (int64_t(1) << 30) || N < kTile || N % kTile != 0 || K < 128 || K % 128 != 0) return CA_EUNSUPPORTED;
  if (ldx < K || ldw < K || ldy < N || ldx % 8 != 0 || ldw % 8 != 0 || ldy % 8 != 0) return CA_EINVAL;
  if (M == 0) return CA_OK;                       // nothing to do
  if (ldx * 2 * kTile >= (int64_t(1) << 31) || ldw * 2 * kTile >= (int64_t(1) << 31)) return CA_EUNSUPPORTED;
  GemmArgs a{};
  a.x = static_cast<const uint16_t*>(x);
  a.w = static_cast<const uint16_t*>(w);
  a.y = static_cast<uint16_t*>(y);
  a.M = int32_t(M); a.N = N; a.K = K;
  a.ldx = ldx; a.ldw = ldw; a.ldy = ldy;
  a.tiles_m = int32_t((M + kTile - 1) / kTile);
  a.tiles_n = N / kTile;
  a.sb_cols = (a.tiles_n + kSbCols - 1) / kSbCols;
  a.n_sb = ((a.tiles_m + kSbRows - 1) / kSbRows) * a.sb_cols;
  const unsigned rounds = unsigned((a.n_sb + 7) / 8);
  if (const int32_t rc = ensure_dynamic_lds(reinterpret_cast<const void*>(gemm_bf16_kernel), kGemmLds, 1); rc != CA_OK)
    return rc;
  hipLaunchKernelGGL(gemm_bf16_kernel, dim3(rounds * 8 * 32), dim3(256), kGemmLds,
                     static_cast<hipStream_t>(stream), a);
  return finish_launch("gemm_bf16.hip");
}

}  // namespace ca
