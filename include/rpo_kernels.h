/*
 * rpo_kernels.h -- building-block entry points of librpo, exported so that the
 * dense contraction can be checked on its own and so that tests can run the whole
 * path through the generic (vector-ALU) kernels as a cross-check of the MFMA ones.
 * Same conventions as rpo.h (caller-owned device buffers, stream as void*, int
 * error codes, rpo_last_error()).
 */
#ifndef RPO_KERNELS_H
#define RPO_KERNELS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* C[M,N] (op)= A[M,K] * W[N,K]^T with fp32 accumulation: the projection y = x W^T
 * used by every linear layer of the decoder (QKV, O, gate/up, down, LM head).
 *   a_dev  device, [M, K] row-major, row stride lda (elements), dtype RPO_F32 / RPO_BF16
 *   w_dev  device, [N, K] row-major, row stride ldw, same dtype
 *   c_dev  device, [M, N] row-major, row stride ldc
 *   epilogue 0: C = result in `dtype`; 1: C = result as fp32; 2: C (fp32) += result
 * bf16 operands with K, lda, ldw multiples of 8 and 16-byte aligned bases run on the
 * matrix cores; anything else on the generic kernel.  Errors: RPO_EINVAL, RPO_EHIP. */
int rpo_gemm_nt(const void *a_dev, int64_t lda, const void *w_dev, int64_t ldw, void *c_dev, int64_t ldc,
                int32_t M, int32_t N, int32_t K, int32_t dtype, int32_t epilogue, void *stream);

/* Process-wide kernel selection: 0 = fastest available kernel for the shape (default),
 * 1 = generic vector-ALU kernels for GEMM and attention regardless of shape.
 * Not thread-safe against concurrent compute calls.  Errors: RPO_EINVAL. */
int rpo_set_kernel_path(int path);

#ifdef __cplusplus
}
#endif
#endif /* RPO_KERNELS_H */
