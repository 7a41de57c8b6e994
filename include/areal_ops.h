/*
 * areal_ops.h -- single-kernel entry points of the library, for parity tests
 * and tuning sweeps of one kernel in isolation.  They launch exactly the
 * kernels the generation calls of areal.h launch; all pointers are device
 * pointers, the work is enqueued on `hip_stream` and not waited for.
 */
#ifndef AREAL_OPS_H
#define AREAL_OPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The projection GEMM of the decoder blocks (the dense contractions of the
 * policy forward pass, Section 2 "LLM Training and Inference"):
 *   mode 0: C float32 [M,N]  = A W0^T
 *   mode 1: C float32 [M,N] += A W0^T
 *   mode 2: C half    [M,N]  = silu(A W0^T) * (A W1^T)      (W0 gate, W1 up)
 * A half [M,K], W0/W1 half [N,K] (IEEE fp16), row-major, 16-byte aligned, K % 8 == 0.
 * cfg = tile configuration 0 .. areal_op_gemm_num_configs()-1, or -1 for the
 * library's own choice; splits = K split (>1 accumulates with float32 atomics:
 * in mode 0 C must be zero beforehand), or -1 for the library's choice.
 * Returns 0 or AREAL_E_INVAL / AREAL_E_HIP. */
int areal_op_gemm(void* hip_stream, const void* A, const void* W0, const void* W1, void* C,
                  int32_t M, int32_t N, int32_t K, int32_t mode, int32_t cfg, int32_t splits);
int areal_op_gemm_num_configs(void);
/* The tile configuration and K split the library takes for a product of this
 * shape and mode (host only, no GPU call).  0 or AREAL_E_INVAL. */
int areal_op_gemm_choose(int32_t M, int32_t N, int32_t K, int32_t mode, int32_t* cfg_out,
                         int32_t* splits_out);

/* Calibration for the roofline of the streaming kernels (Section 3.2: decoding is
 * memory-IO bound): a kernel that reads `bytes` (multiple of 16, device, 16-byte
 * aligned) from `src` and does nothing else, launched like the decode kernels
 * (one work-group per 64 KiB).  Timed by the caller, it says what bandwidth a
 * read of that size reaches on this device, ramp-up of the launch included.
 * `sink16`: 16 bytes of device memory that may be written.
 * Returns 0 or AREAL_E_INVAL / AREAL_E_HIP (message: areal_last_error(NULL)). */
int areal_op_stream_read(void* hip_stream, const void* src, uint64_t bytes, void* sink16);

#ifdef __cplusplus
}
#endif
#endif /* AREAL_OPS_H */
