/*
 * mfma_probe.h -- C ABI of libssmm_probe.so, a measurement aid that bench.py loads (no passage of
 * the paper; it is not part of the SSMM library and prices the roofline its kernels are read
 * against).  Times iters x 8 back-to-back matrix instructions per wavefront, one wavefront per SIMD
 * on every CU, after one untimed launch of the same length.
 *   operands    in   device, at least ssmm_probe_operand_bytes() bytes: 8 sets x 64 lanes of A
 *                    operands (16 bytes), B operands (32 bytes; the dense instruction takes the
 *                    first 16) and index registers (4 bytes) -- their bits set the power the
 *                    matrix pipes draw and with it the clock the chip sustains
 *   idle_slots       0, 1, 2 or 4: s_nop 7 (8 wait states) behind every MFMA; -4: none, and four
 *                    consecutive MFMAs share their B operand (the order of the SSMM kernels)
 *   kind             the instruction, one of the constants below
 *   sink        out  device, one float (never written in practice; keeps the sums alive)
 *   ms_out      out  host: duration of the timed launch in milliseconds
 * Synchronises the stream.  Returns 0, or -1 (argument), -3 (operand buffer too small), -4 (HIP).
 */
#ifndef SSMM_MFMA_PROBE_H
#define SSMM_MFMA_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SSMM_PROBE_SMFMAC_32X32X32 = 0, /* v_smfmac_f32_32x32x32_bf16: 2*32*32*32 dense-equivalent FLOPs */
  SSMM_PROBE_SMFMAC_16X16X64 = 1, /* v_smfmac_f32_16x16x64_bf16: 2*16*16*64 dense-equivalent FLOPs */
  SSMM_PROBE_MFMA_32X32X16 = 2    /* v_mfma_f32_32x32x16_bf16 (dense): 2*32*32*16 FLOPs */
};

size_t ssmm_probe_operand_bytes(void);
int ssmm_probe_mfma(const void* operands, size_t operand_bytes, int iters, int idle_slots, int kind, float* sink,
                    float* ms_out, void* stream);

/*
 * Streaming read of `bytes` (>= 1 MiB, 16-byte aligned) of device memory by blocks_per_cu (1..8) blocks of
 * 256 threads per compute unit, each thread with in_flight (1, 2, 4 or 8) 16-byte loads outstanding; one
 * untimed pass, then one timed.  A buffer far larger than the 256 MB memory-side cache measures HBM.
 *   sink    out  device, 16 bytes (never written in practice; keeps the loads alive)
 *   ms_out  out  host: duration of the timed pass in milliseconds (bytes actually read: the largest multiple
 *                of in_flight * 4096 bytes that fits)
 * Synchronises the stream.  Returns 0, -1 (argument) or -4 (HIP).
 */
int ssmm_probe_hbm_read(const void* buf, size_t bytes, int blocks_per_cu, int in_flight, void* sink, float* ms_out,
                        void* stream);

#ifdef __cplusplus
}
#endif
#endif
