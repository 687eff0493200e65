// Measurement aid, not part of the method and not part of libssmm.so (it builds into
// libssmm_probe.so, which only bench.py loads): the rate at which the matrix pipes of the device
// sustain back-to-back matrix instructions, one wavefront per SIMD on every CU, with operands the
// caller supplies.  Three instructions, same operand registers: the sparse MFMA of the SSMM kernels
// (v_smfmac_f32_32x32x32_bf16), the other sparse shape (v_smfmac_f32_16x16x64_bf16) and the dense
// MFMA a kernel working on expanded tiles would issue (v_mfma_f32_32x32x16_bf16).  The rate depends
// on the operand bits (the chip is power-limited under matrix load) and on how many issue slots stay
// idle between two MFMAs, which is what the roofline of the SSMM kernels has to be read against.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mfma_probe.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 probe_a_t;
typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 probe_b_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float probe_c16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float probe_c4_t;

constexpr int kProbeSets = 8;                                     // operand sets (and accumulators) per wavefront
constexpr size_t kProbeBytes = kProbeSets * 64 * (16 + 32 + 4);   // A, B and index registers of 64 lanes

// KIND: the instruction (mfma_probe.h).  IDLE: s_nop 7 (8 wait states = 32 cycles of the wave's
// issue) behind every MFMA.  SHARE_B: four consecutive MFMAs take the same B operand (the order of
// the SSMM kernels: the token-tile operand stays while the weight streams change).
template <int KIND, int IDLE, bool SHARE_B>
__global__ void __launch_bounds__(256) probe_mfma_kernel(const char* __restrict__ operands, int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  probe_a_t a[kProbeSets];
  probe_b_t b[kProbeSets];
  uint32_t ix[kProbeSets];
  probe_c16_t acc[kProbeSets];   // the 16x16 shape uses the first four registers of each
  probe_c4_t acc4[kProbeSets];
#pragma unroll
  for (int m = 0; m < kProbeSets; m++) {
    a[m] = *(const probe_a_t*)(operands + (size_t)(m * 64 + lane) * 16);
    b[m] = *(const probe_b_t*)(operands + kProbeSets * 64 * 16 + (size_t)(m * 64 + lane) * 32);
    ix[m] = *(const uint32_t*)(operands + kProbeSets * 64 * 48 + (size_t)(m * 64 + lane) * 4);
#pragma unroll
    for (int r = 0; r < 16; r++) acc[m][r] = 0.f;
#pragma unroll
    for (int r = 0; r < 4; r++) acc4[m][r] = 0.f;
  }
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int m = 0; m < kProbeSets; m++) {
      const int mb = SHARE_B ? m / 4 * 4 : m;
      if (KIND == SSMM_PROBE_SMFMAC_32X32X32)
        asm volatile("v_smfmac_f32_32x32x32_bf16 %0, %1, %2, %3" : "+a"(acc[m]) : "v"(a[m]), "v"(b[mb]), "v"(ix[m]));
      if (KIND == SSMM_PROBE_SMFMAC_16X16X64)
        asm volatile("v_smfmac_f32_16x16x64_bf16 %0, %1, %2, %3" : "+a"(acc4[m]) : "v"(a[m]), "v"(b[mb]), "v"(ix[m]));
      if (KIND == SSMM_PROBE_MFMA_32X32X16) {   // dense: the B operand is the first half of the 16-element register set
        const probe_a_t bd = __builtin_shufflevector(b[mb], b[mb], 0, 1, 2, 3, 4, 5, 6, 7);
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[m]) : "v"(a[m]), "v"(bd));
      }
#pragma unroll
      for (int q = 0; q < IDLE; q++) asm volatile("s_nop 7");
    }
  }
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");   // the last MFMAs retire before their results are read
  float s = 0.f;
#pragma unroll
  for (int m = 0; m < kProbeSets; m++) {
#pragma unroll
    for (int r = 0; r < 16; r++) s += acc[m][r];
#pragma unroll
    for (int r = 0; r < 4; r++) s += acc4[m][r];
  }
  if (s == 12345.678f) sink[0] = s;   // keeps the accumulators alive
}

template <int KIND>
void launch_kind(int idle_slots, unsigned blocks, hipStream_t s, const char* p, int n, float* sink) {
  if (idle_slots == 0) hipLaunchKernelGGL((probe_mfma_kernel<KIND, 0, false>), dim3(blocks), dim3(256), 0, s, p, n, sink);
  if (idle_slots == 1) hipLaunchKernelGGL((probe_mfma_kernel<KIND, 1, false>), dim3(blocks), dim3(256), 0, s, p, n, sink);
  if (idle_slots == 2) hipLaunchKernelGGL((probe_mfma_kernel<KIND, 2, false>), dim3(blocks), dim3(256), 0, s, p, n, sink);
  if (idle_slots == 4) hipLaunchKernelGGL((probe_mfma_kernel<KIND, 4, false>), dim3(blocks), dim3(256), 0, s, p, n, sink);
  if (idle_slots == -4) hipLaunchKernelGGL((probe_mfma_kernel<KIND, 0, true>), dim3(blocks), dim3(256), 0, s, p, n, sink);
}

}  // namespace

extern "C" size_t ssmm_probe_operand_bytes(void) { return kProbeBytes; }

extern "C" int ssmm_probe_mfma(const void* operands, size_t operand_bytes, int iters, int idle_slots, int kind, float* sink,
                               float* ms_out, void* stream) {
  if (!operands || !sink || !ms_out || iters < 1 || iters > (1 << 24)) return -1;
  if (operand_bytes < kProbeBytes) return -3;
  if (idle_slots != 0 && idle_slots != 1 && idle_slots != 2 && idle_slots != 4 && idle_slots != -4) return -1;
  if (kind != SSMM_PROBE_SMFMAC_32X32X32 && kind != SSMM_PROBE_SMFMAC_16X16X64 && kind != SSMM_PROBE_MFMA_32X32X16) return -1;
  hipStream_t s = (hipStream_t)stream;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return -4;
  const unsigned blocks = (unsigned)cus;   // four wavefronts = one per SIMD on every CU
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -4;
  auto launch = [&](int n) {
    const char* p = (const char*)operands;
    if (kind == SSMM_PROBE_SMFMAC_32X32X32) launch_kind<SSMM_PROBE_SMFMAC_32X32X32>(idle_slots, blocks, s, p, n, sink);
    if (kind == SSMM_PROBE_SMFMAC_16X16X64) launch_kind<SSMM_PROBE_SMFMAC_16X16X64>(idle_slots, blocks, s, p, n, sink);
    if (kind == SSMM_PROBE_MFMA_32X32X16) launch_kind<SSMM_PROBE_MFMA_32X32X16>(idle_slots, blocks, s, p, n, sink);
  };
  int st = 0;
  launch(iters);   // brings the chip to the clock it holds under this load
  if (hipEventRecord(e0, s) != hipSuccess) st = -4;
  launch(iters);
  if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) st = -4;
  if (hipGetLastError() != hipSuccess) st = -4;
  float ms = 0.f;
  if (st == 0 && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) st = -4;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *ms_out = ms;
  return st;
}
