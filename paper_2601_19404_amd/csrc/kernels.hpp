// Launchers of the HIP kernels behind the RPO rollout C ABI (host-callable).
// Every launcher validates nothing: callers (rpo_api.hip) check shapes first.
#pragma once

#include "common.hpp"

namespace rpo {

enum DType : int { kF32 = 0, kBF16 = 1 };

inline size_t dtype_size(int dt) { return dt == kF32 ? 4 : 2; }

// One packed sequence of token rows inside a chunk pushed through the layers.
struct SeqDesc {
    int row_start;  // first row of the sequence in the packed row buffer
    int n_rows;     // rows of this sequence in the buffer
    int pos0;       // absolute position (0-based over prompt || answer) of its first row
    int table_off;  // offset (in int32) of its page table inside the table array
};

// ---- GEMM: C[M,N] (op)= A[M,K] * W[N,K]^T, fp32 accumulation -----------------
enum Epilogue : int {
    kEpiStore = 0,     // C has the input dtype
    kEpiStoreF32 = 1,  // C is fp32
    kEpiAddF32 = 2,    // C is fp32 and is accumulated into (residual stream)
    kEpiSwiglu = 3,    // W = [gate rows; up rows] (N = 2F): C[M, F] = silu(A Wg^T) * (A Wu^T), input dtype
    kEpiPartial = 4,   // internal: fp32 partial sums of one K split
    kEpiRope = 5,      // internal: rotary embedding + KV page write from the accumulators (QKV projection)
    kEpiLse = 8,       // internal: no C; per row and 64-column block the maximum and the sum of
                       // 2^((z - max) k2), plus the value at the row's target column (LM head of the
                       // log-prob pass: the logits never reach memory)
    kEpiLogitsMax = 9, // internal: kEpiStoreF32 that also leaves each row's maximum per 64-column block
};
// Outputs of the kEpiLse epilogue (GemmArgs::lse): see launch_lse_combine for what follows.
struct LseFuse {
    float* part = nullptr;          // [M, blocks, 2] (max, sum) per row and column block
    float* target_logit = nullptr;  // [M] z[row, target[row]]
    const int32_t* target = nullptr;  // [M] column ids (out of range: target_logit untouched)
    float k2 = 0.f;                 // log2(e) / temperature
    int blocks = 0;                 // filled in by the launch: column blocks per row
};
struct RopeKvArgs;
struct GemmArgs {
    const void* A;
    int64_t lda;
    const void* W;
    int64_t ldw;
    void* C;
    int64_t ldc;
    int M, N, K;
    int dtype;     // element type of A and W
    int epilogue;  // Epilogue
    int path;      // 0 = pick, 1 = force the generic (non-MFMA) kernel
    void* ws;      // fp32 scratch for K-split partial sums (may be null: no splitting)
    size_t ws_bytes;
    // Optional, with kEpiAddF32 only: after C += A W^T, also write the RMS-normalised rows
    // norm_out[m, :] = C[m, :] / sqrt(mean(C[m, :]^2) + norm_eps) * norm_gain (input dtype, row
    // stride N).  Fused into the K-split reduction when the problem is split.
    const void* norm_gain = nullptr;
    void* norm_out = nullptr;
    float norm_eps = 0.f;
    // Optional, with kEpiStore only (the QKV projection): after C = A W^T, rotate q and k of every
    // row and write k, v into the KV pages (rope->qkv must be C).  Fused into the K-split
    // reduction when the problem is split (the rotation then reads the fp32 sums: one rounding).
    const RopeKvArgs* rope = nullptr;
    // Optional, with kEpiStoreF32 only (the LM head of the log-prob pass): if the launch can fuse the
    // log-sum-exp (gemm_fuses_lse), C is not written and *lse receives the partial results instead.
    LseFuse* lse = nullptr;
    // Optional, with kEpiStoreF32 only (the LM head of a decode step): if the launch can (gemm_fuses_max),
    // it also writes block_max->part[row, block] = max of the row over that column block.
    LseFuse* block_max = nullptr;
};
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);
// Whether launch_gemm would honour GemmArgs::lse for these arguments, and with how many column
// blocks per row (0 = it would write C as usual).
int gemm_fuses_lse(const GemmArgs& a);
int gemm_fuses_max(const GemmArgs& a);
// out[r] = max_b part[r, b]  /  out[r] = max_i logits[r, i]
hipError_t launch_row_max_blocks(const float* part, int blocks, float* out, int rows, hipStream_t s);
hipError_t launch_row_max(const float* logits, int64_t row_stride, int vocab, float* out, int rows, hipStream_t s);

// Practical-ceiling probes (probes.hip): a plain copy (GB/s, read + write) and an MFMA issue loop.
hipError_t probe_copy(const void* src, void* dst, size_t bytes, int reps, double* gbps, hipStream_t s);
hipError_t probe_mfma(float* scratch, int iters, int reps, double* tflops, hipStream_t s);

// Identifiers of the kernels whose launches can be timed (rpo_profile_start).
enum KernelId : int {
    kKidNone = 0,
    // tile shapes of gemm_dma_kernel / gemm_mfma_kernel <BM, BN, waves along M, waves along N>
    kKidGemm256 = 1,        // <256,256,2,4> (many-tile problems)
    kKidGemm128 = 3,        // <128,128,2,2> (decode-sized problems with a deep K, K split)
    kKidGemm64 = 4,         // <64,128,1,2>  (the same for M <= 64)
    kKidGemm32 = 5,         // <32,128,1,4>  (decode QKV projection: one head per tile, no K split)
    kKidGemm64x64 = 6,      // <64,64,2,2>   (decode-sized problems with a shallow K, no K split)
    kKidGemmGeneric = 7,
    kKidGemm256x192 = 11,   // <256,192,4,2> (large M, narrow N: fewer idle CUs in the last round)
    kKidAttnDecode = 8,     // attn_decode_mfma_kernel
    kKidAttnChunk = 9,      // attn_chunk_mfma_kernel
    kKidSample = 10,        // sample_kernel
    kKidGemm256Swiglu = 12, // <256,256,2,4> with the fused SwiGLU epilogue (gate/up of prefill / log-prob chunks)
    kKidGemm256x160 = 13,   // <256,160,4,1> fused SwiGLU only (decode gate/up: one round of workgroups on more CUs)
    kKidCount = 14,
};
// Which kernel launch_gemm picks for these arguments.
int gemm_kernel_id(const GemmArgs& a);
// Bytes of fp32 K-split partial sums launch_gemm would write for these arguments if the
// workspace were unlimited (0 = the problem is not split along K); a.ws / a.ws_bytes are ignored.
size_t gemm_splitk_scratch_bytes(const GemmArgs& a);

// ---- elementwise ---------------------------------------------------------------
// x[r, :] = embed[tokens[idx(r)], :] as fp32, idx(r) = tok_index ? tok_index[r] : r;
// out-of-range ids and idx(r) < 0 give a zero row.
hipError_t launch_embed(const int32_t* tokens, const int32_t* tok_index, const void* embed, int dtype,
                        int vocab, int d, float* x, int rows, hipStream_t s);
// h[r, :] = x[src(r), :] / sqrt(mean(x^2) + eps) * gain, src(r) = row_idx ? row_idx[r] : r.
// x fp32, gain and h in `dtype`.
hipError_t launch_rmsnorm(const float* x, const int32_t* row_idx, const void* gain, int dtype, int d,
                          float eps, void* h, int rows, hipStream_t s);
// act[r, j] = silu(gu[r, j]) * gu[r, F + j]
hipError_t launch_swiglu(const void* gu, int dtype, int F, void* act, int rows, hipStream_t s);
// dst[r, :] = src[row_idx[r], :] (fp32 rows of width d)
hipError_t launch_gather_rows(const float* src, const int32_t* row_idx, int d, float* dst, int rows,
                              hipStream_t s);

// Rotate q and k of every row by its position, write k and v into the row's KV page.
struct RopeKvArgs {
    void* qkv;  // [rows, (Hq + 2 Hkv) dh], q rotated in place
    int dtype;
    int rows;
    int Hq, Hkv, dh;
    const float* rope;      // [max_pos, dh/2, 2] (cos, sin)
    const int32_t* row_seq;  // row -> sequence index (< 0: a padding row, nothing is written), or NULL: sequence = row
    const SeqDesc* seqs;
    int pos_add;             // added to every position (decode step)
    int single_row = 0;      // 1: every row is THE row of its sequence (position pos0 + pos_add) wherever it
                             // sits in the row buffer (decode step over a compacted batch)
    const int32_t* tables;
    const uint8_t* active;  // per row, or NULL
    void* kv_pool;
    KvGeom geom;
    int layer;
};
hipError_t launch_rope_kv(const RopeKvArgs& a, hipStream_t s);

// Copy the partially filled last prefix page of each group into the first private
// page of each of its rollouts, all layers.  src_page/dst_page per rollout; src < 0 = nothing.
hipError_t launch_fork_copy(void* kv_pool, int dtype, KvGeom geom, int n_layers, const int32_t* src_page,
                            const int32_t* dst_page, int n_rollouts, hipStream_t s);

// ---- attention over the paged cache --------------------------------------------
// Causal attention of packed rows: row i of sequence s (position pos0 + i + pos_add) sees
// positions [0, pos0 + i + pos_add] of that sequence's pages.
struct AttnArgs {
    const void* q;  // [rows, q_stride]; head h at column h * dh
    int64_t q_stride;
    void* out;  // [rows, Hq * dh]
    int dtype;
    int rows;
    int Hq, Hkv, dh;
    const int32_t* row_seq;  // or NULL: sequence = row; < 0: a padding row (skipped)
    int single_row = 0;      // as in RopeKvArgs
    const SeqDesc* seqs;
    int n_seqs;
    int max_seq_rows;  // largest n_rows among seqs (grid sizing)
    int pos_add;
    const int32_t* tables;
    const uint8_t* active;  // per row, or NULL
    const void* kv_pool;
    KvGeom geom;
    int layer;
    float scale;
    int path;  // 0 = pick, 1 = force generic
};
hipError_t launch_attn_chunk(const AttnArgs& a, hipStream_t s);
// Whether the MFMA attention kernels take these arguments.
bool attn_uses_mfma(const AttnArgs& a);

// Decode attention with a shared prefix: rollout rows r = g * G + i, one new query row
// each; rows of a group share the group's first shared_pages[g] pages.
struct DecodeAttnArgs {
    AttnArgs base;               // seqs = per-rollout descriptors (n_rows = 1); base.rows = query rows
    int n_rollouts;              // rollout rows r = g * G + i covered (= base.rows unless compacted)
    const int32_t* row_of = nullptr;  // compacted batch: rollout -> query / output row, < 0 = finished
                                      // (base.row_seq is then the inverse map); NULL: row = rollout
    int G;
    const int32_t* shared_pages;  // per group: full prefix pages shared by its rollouts
    int max_shared_pages;
    int max_own_pages;  // private pages any rollout can hold at this step
    float* partial;     // split-KV scratch
    size_t partial_floats;
};
hipError_t launch_attn_decode(const DecodeAttnArgs& a, hipStream_t s);
size_t attn_decode_partial_floats(int rows, int Hq, int dh, int max_shared_pages);

// ---- sampling, log-probs, advantages -------------------------------------------
struct SampleArgs {
    const float* logits;
    int n_logit_rows, vocab;
    int64_t row_stride;
    const int32_t* row_map;
    int n_out_rows;
    float inv_t;
    uint64_t seed;
    const uint64_t* seq_id;
    uint32_t step;
    int32_t* tokens_out;
    float* logprob_out;
    int eos_id;          // < 0: no end-of-sequence token
    uint8_t* active;     // in/out per output row, or NULL: all rows live
    int32_t* lengths;    // in/out per output row (tokens generated so far), or NULL
    const float* row_max = nullptr;  // per logits row: its maximum, or NULL: the kernel finds it
};
hipError_t launch_sample(const SampleArgs& a, hipStream_t s);

// out[r] = logits[r, target[r]] * inv_t - logsumexp(logits[r, :] * inv_t)
// out[r] = (target_logit[r] - M) / T - ln(sum_b part[r, b].sum * 2^((part[r, b].max - M) k2)),
// M = max_b part[r, b].max: the log-softmax value of the target from the pieces kEpiLse leaves.
// (NaN for a target outside [0, vocab))
hipError_t launch_lse_combine(const float* part, int blocks, const float* target_logit, const int32_t* target,
                              int vocab, float inv_t, float* out, int rows, hipStream_t s);
hipError_t launch_lse_gather(const float* logits, int64_t row_stride, int vocab, const int32_t* target,
                             float inv_t, float* out, int rows, hipStream_t s);

// ---- experience cache (cache.hip) ----------------------------------------------
hipError_t launch_cut_pack(const int32_t* prompts, int64_t prompt_stride, const int32_t* prompt_len,
                           const int32_t* pool, int64_t pool_stride, const int32_t* question,
                           const int32_t* cu_len, int n_groups, int32_t* out, hipStream_t s);
hipError_t launch_cache_update(int32_t* pool, int64_t pool_stride, int32_t* answer_len, const int32_t* question,
                               const int32_t* m,
                               const int32_t* tokens, int64_t tok_stride, const int32_t* lengths,
                               const float* rewards, const float* u, const int32_t* g_prime, int n_groups, int G,
                               float eps, int32_t* chosen_out, hipStream_t s);

hipError_t launch_objective(const float* lp_new, const float* lp_old, const float* lp_ref, const int32_t* cu,
                            const float* adv, int n_groups, int G, float eps_clip, float beta, float* tok_out,
                            double* per_rollout, float* j_out, hipStream_t s);
hipError_t launch_shape_rewards(const float* rewards, const int32_t* lengths, int n_groups, int G, float alpha,
                                float lo, float hi, float* out, hipStream_t s);
// Compaction of a decode batch: live[c] = c-th rollout row r < n_rows with active[r] != 0 (in
// increasing r; -1 for c >= their number), row_of[r] = c or -1, and their number to *count_dev
// and, if given, as (generation << 32 | number) to *mailbox (device address of mapped host memory).
hipError_t launch_compact_rows(const uint8_t* active, int n_rows, int32_t* live, int32_t* row_of,
                               int32_t* count_dev, uint64_t* mailbox, uint32_t generation, hipStream_t s);
hipError_t launch_advantages(const float* rewards, int n_groups, int G, int ddof, float eps, float* adv,
                             hipStream_t s);

}  // namespace rpo
