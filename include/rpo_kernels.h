/*
 * rpo_kernels.h -- building-block entry points of librpo, exported so that the
 * dense contraction can be checked on its own and so that tests can run the whole
 * path through the generic (vector-ALU) kernels as a cross-check of the MFMA ones.
 * Same conventions as rpo.h (caller-owned device buffers, stream as void*, int
 * error codes, rpo_last_error()).
 */
#ifndef RPO_KERNELS_H
#define RPO_KERNELS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* C[M,N] (op)= A[M,K] * W[N,K]^T with fp32 accumulation: the projection y = x W^T
 * used by every linear layer of the decoder (QKV, O, gate/up, down, LM head).
 *   a_dev  device, [M, K] row-major, row stride lda (elements), dtype RPO_F32 / RPO_BF16
 *   w_dev  device, [N, K] row-major, row stride ldw, same dtype
 *   c_dev  device, [M, N] row-major, row stride ldc
 *   epilogue 0: C = result in `dtype`; 1: C = result as fp32; 2: C (fp32) += result;
 *            3: SwiGLU: W rows are [gate (F rows); up (F rows)], N = 2F, and
 *               C[M, F] = silu(A Wgate^T) * (A Wup^T) in `dtype` (ldc >= F)
 *   ws_dev   device scratch for K-split partial sums, ws_bytes long, or NULL / 0: skinny
 *            problems are then not split along K (same result, fewer busy CUs)
 * bf16 operands with K, lda, ldw multiples of 8 and 16-byte aligned bases run on the
 * matrix cores (SwiGLU also needs F a multiple of 32); anything else on the generic
 * kernel.  Errors: RPO_EINVAL, RPO_EHIP. */
int rpo_gemm_nt(const void *a_dev, int64_t lda, const void *w_dev, int64_t ldw, void *c_dev, int64_t ldc,
                int32_t M, int32_t N, int32_t K, int32_t dtype, int32_t epilogue, void *ws_dev,
                size_t ws_bytes, void *stream);

/* The shared-prefix decode attention of ONE layer on its own (the kernel rpo_decode_step runs
 * between the QKV and the output projection), so that it can be checked against a plain
 * softmax(q K^T / sqrt(dh)) V and profiled alone.  For rollout rows [0, n_rows) of a forked batch:
 * one query row per rollout attends to [the group's shared prefix pages || the rollout's private
 * pages], i.e. to positions [0, prefix_len(group) + n_suffix) of whatever keys / values the batch's
 * pages hold for `layer` (the prefix after rpo_prefill_prefix + rpo_kv_fork; private positions
 * that no decode step or log-prob pass has written hold zeros).
 *   q_dev      device, [n_rows, n_q_heads * head_dim], model dtype, already rotated
 *   n_suffix   private tokens each rollout sees, 0..max_suffix
 *   active_dev device uint8 [n_rows] or NULL; rows with 0 are skipped (their output row is untouched)
 *   out_dev    device, [n_rows, n_q_heads * head_dim], model dtype
 * Uses the batch's workspace (attention partials): not concurrently with other calls on the batch.
 * Errors: RPO_ESTATE unless forked; RPO_EINVAL. */
struct rpo_batch;
int rpo_attn_decode(struct rpo_batch *b, int32_t layer, const void *q_dev, int32_t n_rows, int32_t n_suffix,
                    const uint8_t *active_dev, void *out_dev, void *stream);

/* rpo_gemm_nt for callers that cannot allocate or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same contraction, kernels and
 * results, with the K-split partial sums in a fixed 16 MiB device array that belongs to the
 * library (one copy per GPU, held until the process ends).  Allocates nothing, on the host or the
 * device.  Arguments as rpo_gemm_nt.  A problem whose K split needs more than 16 MiB of partial
 * sums (splits * M * N * 4 bytes; only skinny problems with a deep K are split) is rejected with
 * RPO_ENOMEM and nothing is enqueued.  All calls on one GPU share the array: calls that may run
 * concurrently on one GPU (different streams, different threads) race on it; calls on one
 * stream are safe.  Nothing in the array needs clearing between calls (every partial sum is
 * written before it is read).  Errors: RPO_EINVAL, RPO_ENOMEM, RPO_EHIP. */
int rpo_gemm_nt_noalloc(const void *a_dev, int64_t lda, const void *w_dev, int64_t ldw, void *c_dev, int64_t ldc,
                        int32_t M, int32_t N, int32_t K, int32_t dtype, int32_t epilogue, void *stream);

/* Practical ceilings of the GPU the library runs on, for roofline reports: the rate of a plain
 * device-to-device copy of `bytes` bytes (read + write counted, GB/s, best of three launches) and
 * of a back-to-back bf16 32x32x16 MFMA issue loop with changing operands (TFLOP/s, two workgroups
 * of four waves per CU, about 0.1 s, best of two).
 *   src_dev, dst_dev  device, `bytes` long each (a multiple of 16, at least 1 MiB), not overlapping
 *   scratch_dev       device, 512 * 256 floats, overwritten
 *   copy_gbps, mfma_tflops  host, results
 * Synchronises the stream.  Errors: RPO_EINVAL, RPO_EHIP. */
int rpo_probe_peaks(const void *src_dev, void *dst_dev, size_t bytes, float *scratch_dev, double *copy_gbps,
                    double *mfma_tflops, void *stream);

/* TEST AND TUNING SWITCH, process-wide: 0 = fastest available kernel for the shape (default, and
 * the only value a product run uses),
 * 1 = generic vector-ALU kernels for GEMM and attention regardless of shape (the tests run whole
 *     rollouts through them as a cross-check of the MFMA kernels),
 * 2 = MFMA GEMM with register-staged LDS fills instead of direct-to-LDS loads (the fallback
 *     used when K is not a multiple of 64; selectable so that the tests reach it at any K),
 * 16 + k (k = 1, 3..6, 11) = MFMA GEMM with the fixed tile shape of kernel id k, so that the tests
 *     can force every tile shape onto one problem (attention as in 0).
 * Unsynchronised: set it from the thread that issues the compute calls, between calls.
 * Errors: RPO_EINVAL. */
int rpo_set_kernel_path(int path);

/* Per-kernel timing for roofline reports.  rpo_profile_start(kernel_id, every) makes every
 * `every`-th later launch of that kernel (the 1st, the every+1-th, ...; process-wide, any stream)
 * bracketed by a pair of HIP events recorded on the launch stream; several kernel ids may be
 * timed at once.  rpo_profile_stop(kernel_id, ...) waits for that kernel's last event and returns
 * the number of bracketed launches, their summed event time in milliseconds, and their summed
 * ALGORITHMIC flops and bytes as the library counts them (GEMM: 2MNK flops, operands + result
 * bytes; decode attention: K/V bytes with a group's shared prefix counted once per group;
 * sampler: the logits rows read once).  Kernel ids:
 * (MFMA GEMM tile shapes <BM, BN, waves along M, waves along N>)
 *   1  <256,256,2,4> (prefill-sized problems and wide decode projections), every epilogue but SwiGLU
 *   12 <256,256,2,4> with the fused SwiGLU epilogue: the gate/up projection of prefill and
 *      log-prob chunks, one instantiation, the heaviest kernel of a rollout step
 *   3  <128,128,2,2> (decode-sized problems, deep K)   4  <64,128,1,2> (the same for M <= 64)
 *   5  <32,128,1,4> / <64,128,1,4> (decode QKV projection: rotary embedding and KV page write in
 *      the epilogue; 64 rows once the 32-row tiles would outnumber the CUs)
 *   6  <64,64,2,2> (decode-sized problems, shallow K, no K split)
 *      (all epilogues of a tile shape together; a K-split launch includes its reduction)
 *   11 <256,192,4,2> (large M with a narrow N: fewer idle CUs in the last round of workgroups)
 *   7  gemm_generic_kernel      8  attn_decode_mfma_kernel (+ merge)   9  attn_chunk_mfma_kernel
 *   10 sample_kernel
 * The timing state and rpo_set_kernel_path's switch are process-wide and unsynchronised: use them
 * from the one thread that issues the compute calls, and not while another thread is inside one.
 * Host-side only (event create / record / synchronise).
 * Errors: RPO_EINVAL (unknown id, every < 1, NULL), RPO_EHIP. */
int rpo_profile_start(int kernel_id, int every);
int rpo_profile_stop(int kernel_id, int64_t *n_launches, double *total_ms, double *total_flops,
                     double *total_bytes);

#ifdef __cplusplus
}
#endif
#endif /* RPO_KERNELS_H */
