// MFMA-only microbenchmark: what the matrix pipes of this GPU sustain, at the clock the chip
// actually holds, when every wave issues v_mfma_f32_32x32x16_bf16 back to back and does nothing
// else.  It is the practical ceiling next to which the attention kernel's throughput is read:
// the nominal peak assumes the maximum clock, and under a full MFMA load with operands that
// toggle (random bf16) the chip settles well below it.
//
// One workgroup of 4 waves per CU; a wave runs 8 independent accumulator chains (128 AGPRs), 32
// MFMAs per loop trip, operands fixed in registers.  data_kind 0: all-zero operands (least
// switching), 1: pseudo-random bf16 in [-1, 1) (a hash of lane and register index).
#include <hip/hip_runtime.h>

#include "ca_internal.hpp"

namespace ca {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ uint32_t hash32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// two bf16 in [-1, 1): sign and 7 mantissa bits random, exponent 2^-1 .. 2^-4
__device__ __forceinline__ uint32_t random_bf16_pair(uint32_t seed) {
  const uint32_t h = hash32(seed);
  auto one = [](uint32_t r) {
    const uint32_t sign = (r >> 15) & 1, exp = 123 + ((r >> 7) & 3), man = r & 0x7f;
    return (sign << 15) | (exp << 7) | man;
  };
  return one(h & 0xffff) | (one(h >> 16) << 16);
}

__global__ __launch_bounds__(256, 1) void mfma_peak_kernel(int data_kind, int trips, unsigned long long* probe) {
  u32x4 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t s = (blockIdx.x * 256 + threadIdx.x) * 64 + i * 8 + j;
      a[i][j] = data_kind ? random_bf16_pair(s) : 0u;
      b[i][j] = data_kind ? random_bf16_pair(s + 4) : 0u;
    }
  const unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  asm volatile(
      "s_mov_b32 s36, %8\n"
      "LOOP_%=:\n"
#define CA_MF(acc, A, B) "v_mfma_f32_32x32x16_bf16 a[" acc "], %" A ", %" B ", a[" acc "]\n"
#define CA_EIGHT(A, B0, B1)                                                              \
  CA_MF("0:15", A, B0) CA_MF("16:31", A, B1) CA_MF("32:47", A, B0) CA_MF("48:63", A, B1) \
  CA_MF("64:79", A, B0) CA_MF("80:95", A, B1) CA_MF("96:111", A, B0) CA_MF("112:127", A, B1)
      CA_EIGHT("0", "4", "5") CA_EIGHT("1", "5", "6") CA_EIGHT("2", "6", "7") CA_EIGHT("3", "7", "4")
#undef CA_EIGHT
#undef CA_MF
      "s_sub_u32 s36, s36, 1\n"
      "s_cmp_lg_u32 s36, 0\n"
      "s_cbranch_scc1 LOOP_%=\n"
      "s_nop 15\ns_nop 15\ns_nop 15\n"
      :
      : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(b[0]), "v"(b[1]), "v"(b[2]), "v"(b[3]), "s"(trips)
      : "s36", "scc", "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13",
        "a14", "a15", "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28",
        "a29", "a30", "a31", "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43",
        "a44", "a45", "a46", "a47", "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58",
        "a59", "a60", "a61", "a62", "a63", "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73",
        "a74", "a75", "a76", "a77", "a78", "a79", "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88",
        "a89", "a90", "a91", "a92", "a93", "a94", "a95", "a96", "a97", "a98", "a99", "a100", "a101", "a102",
        "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111", "a112", "a113", "a114", "a115",
        "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127");
  const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  if (threadIdx.x == 0) {
    probe[2 * blockIdx.x] = c1 - c0;
    probe[2 * blockIdx.x + 1] = r1 - r0;       // 100 MHz ticks
  }
}

}  // namespace

int32_t run_mfma_microbench(int data_kind, int trips, void* scratch, size_t scratch_bytes, void* stream,
                            double* tflops, double* clock_ghz) {
  int n_cu = 0;
  if (const int32_t rc = device_cu_count(&n_cu); rc != CA_OK) return rc;
  if (scratch_bytes < size_t(n_cu) * 16) return CA_EINVAL;
  auto* probe = static_cast<unsigned long long*>(scratch);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return finish_launch("hipEventCreate");
  hipLaunchKernelGGL(mfma_peak_kernel, dim3(n_cu), dim3(256), 0, s, data_kind, trips / 8 + 1, probe);  // warm-up
  hipEventRecord(e0, s);
  hipLaunchKernelGGL(mfma_peak_kernel, dim3(n_cu), dim3(256), 0, s, data_kind, trips, probe);
  hipEventRecord(e1, s);
  int32_t rc = finish_launch("mfma_peak.hip");
  float ms = 0.f;
  if (rc == CA_OK && (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
    rc = finish_launch("hipEventSynchronize");
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  if (rc != CA_OK) return rc;
  unsigned long long h[2] = {0, 0};
  if (hipMemcpy(h, probe, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return finish_launch("hipMemcpy");
  const double flops = double(n_cu) * 4.0 * double(trips) * 32.0 * (2.0 * 32 * 32 * 16);
  if (tflops) *tflops = flops / (double(ms) * 1e-3) / 1e12;
  if (clock_ghz) *clock_ghz = h[1] ? double(h[0]) / (double(h[1]) / 100e6) / 1e9 : 0.0;
  return CA_OK;
}

}  // namespace ca
