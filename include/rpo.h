/*
 * rpo.h -- C ABI of the RPO suffix-rollout library for AMD MI355X (gfx950).
 *
 * RPO (arXiv 2601.19404, "Reinforcement Fine-Tuning with Partial Reasoning
 * Optimization") replaces full-path rollouts by regeneration of answer
 * suffixes: for a question q_k with cached answer a_k, the last m tokens are
 * dropped and G continuations are sampled from the policy conditioned on
 * q_k || a_k[0:-m] (Sec. 3.2 "Rollout", Eq. 3; Algorithm 1, rollout lines).
 * The G rollouts of a group share that prefix (Sec. 3.4, first paragraph), so
 * the prefix is prefilled ONCE into a paged key/value cache and forked.  After
 * sampling, the per-token log-probabilities of the sampled suffix tokens (the
 * numerator / denominator of the ratio in Eq. 7) and the group-normalised
 * advantages (Eq. 7) are computed.
 *
 * Conventions
 *  - Every pointer argument says "host" or "device".  Device buffers are owned
 *    by the caller (any allocator; the tests use PyTorch-ROCm tensors) and are
 *    BORROWED by the handles for their lifetime.  The library never allocates
 *    or frees device memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Compute calls only enqueue work: no device-to-host copies, no wait for the stream.
 *    rpo_prefill_prefix, rpo_kv_fork and rpo_suffix_logprobs upload a few small integer tables
 *    (page tables, row maps) from ordinary host memory with hipMemcpyAsync: the runtime may hold
 *    the calling thread until such a copy is staged.  rpo_decode_step, rpo_sample and the
 *    stateless calls upload nothing.  Host arrays passed to a call are consumed before it returns.
 *  - All matrices are row-major.  Projection weights are [out_features,
 *    in_features] (y = x W^T).  Activations / weights are fp32 (RPO_F32) or
 *    bfloat16 (RPO_BF16); logits, log-probs, rewards and advantages are fp32.
 *  - Return value: RPO_OK or a negative error code; rpo_last_error() returns a
 *    thread-local description of the last failure.  Nothing aborts, nothing
 *    throws across the boundary.  Arguments are validated on the host before
 *    anything is enqueued; a failing call enqueues nothing.
 *  - There is no CPU fallback: without a gfx950 device every compute call fails
 *    with RPO_EHIP.
 */
#ifndef RPO_H
#define RPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { RPO_OK = 0, RPO_EINVAL = -1, RPO_ESTATE = -2, RPO_ENOMEM = -3, RPO_EHIP = -4 };
enum { RPO_F32 = 0, RPO_BF16 = 1 };

typedef struct rpo_model rpo_model;
typedef struct rpo_batch rpo_batch;

/* Decoder shape.  The paper names its models (DeepSeek-R1-Distill-Qwen 1.5B / 7B,
 * Sec. 4.1) but not their architecture; this is the standard pre-norm decoder of
 * that family: RMSNorm (eps inside the root), rotary embedding with half-split
 * pairs (i, i + head_dim/2) and angle pos * rope_base^(-2i/head_dim), grouped-query
 * causal attention scaled by 1/sqrt(head_dim) (query head h reads KV head
 * h / (n_q_heads / n_kv_heads)), SwiGLU, no biases, untied LM head. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rope_base, rms_eps;
    int32_t dtype; /* RPO_F32 or RPO_BF16: storage type of weights, activations and KV */
} rpo_model_desc;

/* Device pointers to the weights, element type desc.dtype.
 *   embed [vocab, d_model]; lm_head [vocab, d_model]; final_norm [d_model]
 *   per layer l (host arrays of n_layers device pointers):
 *   attn_norm[l] [d_model]
 *   wqkv[l]      [(n_q_heads + 2 n_kv_heads) * head_dim, d_model]  rows: q heads, k heads, v heads
 *   wo[l]        [d_model, n_q_heads * head_dim]
 *   ffn_norm[l]  [d_model]
 *   w_gate_up[l] [2 * d_ffn, d_model]   rows: gate, then up
 *   w_down[l]    [d_model, d_ffn]                                                    */
typedef struct {
    const void *embed, *lm_head, *final_norm;
    const void *const *attn_norm, *const *wqkv, *const *wo;
    const void *const *ffn_norm, *const *w_gate_up, *const *w_down;
} rpo_weights;

/* Model handle: copies the descriptor and the pointer tables (host memory only).
 * Errors: RPO_EINVAL on NULL / non-positive sizes / n_q_heads not a multiple of
 * n_kv_heads / odd head_dim / unknown dtype. */
int rpo_model_create(const rpo_model_desc *desc, const rpo_weights *weights, rpo_model **out);
void rpo_model_destroy(rpo_model *m);

/* Sizes of the two caller-provided device buffers of a batch.
 *   n_groups   questions in the batch (one sampling group each)
 *   G          rollouts per group
 *   max_prefix longest q || a[0:-m] in tokens
 *   max_suffix most tokens any rollout appends after the prefix
 *   page_tokens tokens per KV page (a power of two, >= 16; the bf16 MFMA
 *              attention kernels need 64)
 *   max_rows   most token rows pushed through the layers at once (prefill and
 *              log-prob passes are cut into chunks of whole sequences of at most
 *              this many rows; must be >= max_prefix, >= max_suffix, >= n_groups * G)
 * Return 0 on invalid arguments. */
size_t rpo_kv_pool_bytes(const rpo_model *m, int32_t n_groups, int32_t G, int32_t max_prefix,
                         int32_t max_suffix, int32_t page_tokens);
size_t rpo_workspace_bytes(const rpo_model *m, int32_t n_groups, int32_t G, int32_t max_prefix,
                           int32_t max_suffix, int32_t page_tokens, int32_t max_rows);

/* Batch handle over caller-owned device buffers `kv_pool` and `workspace`
 * (256-byte aligned, at least the sizes above; contents need not be initialised).
 * Uploads the rotary table and the page tables on `stream`.
 * Errors: RPO_EINVAL, RPO_ENOMEM (buffers too small), RPO_EHIP. */
int rpo_batch_create(const rpo_model *m, int32_t n_groups, int32_t G, int32_t max_prefix,
                     int32_t max_suffix, int32_t page_tokens, int32_t max_rows,
                     void *kv_pool /*device*/, size_t kv_bytes,
                     void *workspace /*device*/, size_t ws_bytes, void *stream, rpo_batch **out);
void rpo_batch_destroy(rpo_batch *b);

/* Eq. 3, conditioning part: forward q_k || a_k[0:-m] once per group, write its
 * keys/values into the group's pages, return the logits of the last prefix row
 * (they score the first regenerated token).
 *   tokens_dev      device int32, the prefixes packed back to back (sum of lengths)
 *   cu_len_host     host int32 [n_groups + 1], cumulative lengths, cu_len[0] = 0;
 *                   every length in [1, max_prefix]
 *   last_logits_dev device fp32 [n_groups, vocab]
 * Resets the batch to "prefilled, not forked".  Errors: RPO_EINVAL, RPO_EHIP. */
int rpo_prefill_prefix(rpo_batch *b, const int32_t *tokens_dev, const int32_t *cu_len_host,
                       float *last_logits_dev, void *stream);

/* Give each of the G rollouts of every group its own page table: full prefix
 * pages are referenced (shared, never written again), the partially filled last
 * prefix page is copied into the rollout's first private page.  Rollout row
 * r = group * G + i.  Errors: RPO_ESTATE unless called right after prefill. */
int rpo_kv_fork(rpo_batch *b, void *stream);

/* One autoregressive step of Eq. 3's continuation for rollout rows [0, n_rows):
 * consume tokens_dev[r] (the token sampled for position prefix_len + step),
 * append its K/V, return the logits that score the next token.
 *   tokens_dev device int32 [n_rows]
 *   n_rows     leading rows to process, 1..n_groups*G.  Groups finish together
 *              (one m per group), so a caller that orders groups by decreasing m
 *              shrinks n_rows as groups finish.
 *   active_dev device uint8 [n_rows] or NULL (all live).  A row with 0 appends
 *              no K/V; its logits row holds unspecified values.
 *   logits_dev device fp32 [n_rows, vocab]
 *   row_max_out_dev device fp32 [n_rows] or NULL: max_i logits[r, i] of every row (the exact
 *              fp32 maximum; taken in the LM-head epilogue where the kernel allows, so that
 *              rpo_sample need not sweep the row for it).  Unspecified for rows with active 0.
 * The step counter is kept by the batch (all live rows advance together).
 * Errors: RPO_ESTATE before fork or beyond max_suffix; RPO_EINVAL. */
int rpo_decode_step(rpo_batch *b, const int32_t *tokens_dev, int32_t n_rows,
                    const uint8_t *active_dev, float *logits_dev, float *row_max_out_dev, void *stream);

/* rpo_decode_step over a COMPACTED batch, for variable-length rollouts (the paper generates until
 * end-of-sequence or the length cap, Sec. 4.1): rollouts that have finished leave the batch
 * instead of being masked, so the projections and the LM head run on the live rows only.
 * A small kernel lists the live rollouts of rows [0, n_rows) (active != 0) in increasing order;
 * query row c of the step belongs to the c-th of them.
 *   active_dev      device uint8 [n_rows], required (rpo_sample's active_inout_dev)
 *   logits_dev      device fp32 [n_rows, vocab]: row c scores the next token of the c-th live
 *                   rollout; rows beyond the live ones hold unspecified values
 *   row_max_out_dev device fp32 [n_rows] or NULL, indexed like logits_dev
 *   row_of_out_dev  device int32 [n_rows]: logits row of rollout r, -1 if it has finished -- pass it
 *                   to rpo_sample as row_map_dev (with n_logit_rows = *n_logit_rows_out)
 *   n_logit_rows_out host int32: logits rows this step computed.  It is the number of live
 *                   rollouts the device last REPORTED to the host (through a pinned word, without
 *                   any wait), hence an upper bound of the live rows of this step that trails the
 *                   true count by the steps still in flight; 0 once every rollout has finished.
 * Everything else as rpo_decode_step.  Errors: RPO_ESTATE, RPO_EINVAL. */
int rpo_decode_step_compact(rpo_batch *b, const int32_t *tokens_dev, int32_t n_rows, const uint8_t *active_dev,
                            float *logits_dev, float *row_max_out_dev, int32_t *row_of_out_dev,
                            int32_t *n_logit_rows_out, void *stream);

/* Draw one token per output row from softmax(logits / temperature) (the paper
 * samples with a temperature, Sec. 4.1).  Stateless.  The draw is defined through
 * integers so that it does not depend on reduction order (bit-exact contract):
 *   x_i = ((z_i - max z) * (1/T)) * log2(e)            three rounded fp32 operations
 *   q_i = floor(P(x_i - rint x_i) * 2^(rint x_i + 40)), q_i = 0 for x_i < -41, where P is
 *         the degree-7 Taylor polynomial of 2^f with fp32 coefficients evaluated by
 *         Horner's rule with separately rounded fp32 multiplies and adds
 *   u   = Philox4x32-10(counter = (step, seq_id lo, seq_id hi, 0), key = (seed lo, seed hi)),
 *         u = out1 * 2^32 + out0;   t = floor(u * sum(q) / 2^64)
 *   token = smallest k with q_0 + ... + q_k > t
 *   logits_dev  device fp32, n_logit_rows rows of `vocab` values, `row_stride` floats apart
 *   row_map_dev device int32 [n_out_rows] or NULL: output row r reads logits row
 *               row_map[r] (G rollouts drawing their first token from one prefix row)
 *   seq_id_dev  device uint64 [n_out_rows]: Philox stream id of each output row
 *   tokens_out_dev  device int32 [n_out_rows]
 *   logprob_out_dev device fp32 [n_out_rows] or NULL: log softmax(z/T)[token] (fp32 accuracy)
 * Variable-length rollouts (the paper generates until end-of-sequence or the length cap,
 * Sec. 4.1; Eq. 11 needs the response lengths):
 *   eos_id            end-of-sequence token id, or < 0 for none
 *   active_inout_dev  device uint8 [n_out_rows] or NULL.  A row with 0 is finished: nothing is
 *                     drawn, its token is eos_id (0 if none) and its log-prob 0.  A live row that
 *                     draws eos_id is set to 0 (pass the same array to rpo_decode_step).
 *   lengths_inout_dev device int32 [n_out_rows] or NULL: incremented for every live row (the
 *                     end-of-sequence token counts).
 *   row_max_dev       device fp32 [n_logit_rows] or NULL.  If given, row_max_dev[k] MUST equal the
 *                     maximum of logits row k exactly (rpo_decode_step's row_max_out_dev); the
 *                     sampler then skips its own maximum sweep.  A wrong value gives a wrong draw.
 * NaN logits give undefined tokens.  Errors: RPO_EINVAL (sizes, temperature <= 0). */
int rpo_sample(const float *logits_dev, int32_t n_logit_rows, int32_t vocab, int64_t row_stride,
               const int32_t *row_map_dev, int32_t n_out_rows, float temperature, uint64_t seed,
               const uint64_t *seq_id_dev, uint32_t step, int32_t *tokens_out_dev,
               float *logprob_out_dev, int32_t eos_id, uint8_t *active_inout_dev,
               int32_t *lengths_inout_dev, const float *row_max_dev, void *stream);

/* log pi(o_j | q, o_<j) of every suffix token (the quantity the ratio of Eq. 7 is
 * made of), teacher-forced: for each rollout row r the suffix tokens are pushed
 * through the layers against the forked prefix pages as one causal chunk (their
 * K/V land in the rollout's private pages), the LM head runs on the suffix rows
 * only, and log-softmax(logits / temperature) is gathered at the target token.
 * The first suffix token is scored by the group's last prefix row.
 *   suffix_tokens_dev device int32, suffixes packed back to back in row order
 *   cu_suffix_host    host int32 [n_groups*G + 1]; each length in [0, max_suffix]
 *   logprobs_out_dev  device fp32, same packing as the tokens
 * A full re-prefill of every sequence (no sharing) is the same call on a batch
 * created with G = 1 whose "prefix" is each sequence's own prefix.
 * Errors: RPO_ESTATE unless forked; RPO_EINVAL. */
int rpo_suffix_logprobs(rpo_batch *b, const int32_t *suffix_tokens_dev, const int32_t *cu_suffix_host,
                        float temperature, float *logprobs_out_dev, void *stream);

/* Eq. 7: A_i = (R_i - mean) / (std + eps) over each group's G rewards.  ddof 0 =
 * population std (default reading), 1 = sample std.  std == 0 with eps == 0 gives
 * A = 0 for the group.  Sums run left to right in fp64, result rounded to fp32.
 *   rewards_dev device fp32 [n_groups, G]; adv_out_dev device fp32 [n_groups, G]
 * Errors: RPO_EINVAL (NULL, G < 1, ddof not 0/1 or >= G, eps < 0). */
int grpo_advantages(const float *rewards_dev, int32_t n_groups, int32_t G, int32_t ddof, float eps,
                    float *adv_out_dev, void *stream);

/* Forward value of the objective, Eq. 5-7: per token l = min(r A, clip(r, 1 - eps_clip, 1 + eps_clip) A)
 * with r = exp(lp_new - lp_old) (the ratio of Eq. 7) and A the rollout's advantage; per group
 * J = mean_i [ (sum_j l_ij - beta * sum_j (lp_new_ij - lp_ref_ij)) / |o_i| ].  The KL term sits
 * outside the min (Eq. 5) and uses the per-token sample estimate of E[log pi - log pi_ref] (App. B
 * names no estimator).  The log-probs come from rpo_suffix_logprobs under the respective weights.
 *   lp_new_dev, lp_old_dev device fp32, packed per token like rpo_suffix_logprobs' output
 *   lp_ref_dev   same, or NULL when beta == 0
 *   cu_suffix_dev device int32 [n_groups*G + 1] cumulative suffix lengths (DEVICE copy)
 *   adv_dev       device fp32 [n_groups*G] (grpo_advantages' output)
 *   token_out_dev device fp32 packed per token, or NULL
 *   rollout_scratch_dev device fp64 [n_groups*G] scratch; group_out_dev device fp32 [n_groups]
 * Empty responses contribute 0.  Errors: RPO_EINVAL. */
int rpo_objective_forward(const float *lp_new_dev, const float *lp_old_dev, const float *lp_ref_dev,
                          const int32_t *cu_suffix_dev, const float *adv_dev, int32_t n_groups, int32_t G,
                          float eps_clip, float beta, float *token_out_dev, double *rollout_scratch_dev,
                          float *group_out_dev, void *stream);

/* Length-aware reward shaping, Eq. 11 (Sec. 3.4): R_i = clip(r_i / (1 + exp(-alpha (l_ref - len_i))),
 * lo, hi) with l_ref the mean response length of the group; the paper uses lo 0.5, hi 1,
 * alpha 0.01 (Sec. 4.1).  Reading: applied to positive rewards only, r_i <= 0 gives R_i = 0
 * (literally, a wrong answer would be lifted to `lo`).  fp64 arithmetic, result fp32; feed
 * the result to grpo_advantages.
 *   rewards_dev device fp32 [n_groups, G]; lengths_dev device int32 [n_groups, G] (tokens per
 *   response); shaped_out_dev device fp32 [n_groups, G].
 * Errors: RPO_EINVAL (NULL, G < 1, alpha <= 0, lo > hi). */
int rpo_shape_rewards(const float *rewards_dev, const int32_t *lengths_dev, int32_t n_groups, int32_t G,
                      float alpha, float lo, float hi, float *shaped_out_dev, void *stream);

/* Eq. 3, the cut, with the cached answers resident on the device: pack q_k || a_k[0 : c_k] of
 * every question back to back -- the `tokens_dev` that rpo_prefill_prefix takes.  c_k follows
 * from the cumulative prefix lengths: c_k = (cu_len[k+1] - cu_len[k]) - prompt_len of its question.
 *   prompts_dev    device int32 [n_questions, prompt_stride]; prompt_len_dev device int32 [n_questions]
 *   pool_dev       device int32 [n_questions, pool_stride]: the cached answers (Eq. 1-2)
 *   question_dev   device int32 [n_groups] or NULL: row of the prompt / pool arrays that batch group
 *                  k reads (NULL: row k; prompts_dev / prompt_len_dev are indexed the same way).  A
 *                  rollout batch orders its groups by suffix length, the pool keeps question order.
 *   cu_len_dev     device int32 [n_groups + 1] (the same values rpo_prefill_prefix gets on the host)
 *   tokens_out_dev device int32 [cu_len[n_groups]]
 * Errors: RPO_EINVAL.  The caller guarantees c_k <= pool_stride. */
int rpo_cut_pack(const int32_t *prompts_dev, int64_t prompt_stride, const int32_t *prompt_len_dev,
                 const int32_t *pool_dev, int64_t pool_stride, const int32_t *question_dev,
                 const int32_t *cu_len_dev, int32_t n_groups, int32_t *tokens_out_dev, void *stream);

/* Cache update, Sec. 3.3 (the epsilon-greedy rule around Eq. 10) and Algorithm 1, "Update
 * Cache": after a step, question k's cached answer becomes a_k[0 : len_k - m_k] || o, where o is
 * the response the rule selects among the G just sampled: the one with the highest reward when
 * u_k <= eps (ties: lowest index), otherwise response g'_k (Algorithm 1 draws g' over all G).
 * The random numbers are inputs.  In place, on the device: the next rpo_cut_pack reads what this
 * call wrote, no token leaves HBM.
 *   pool_dev       device int32 [n_questions, pool_stride], updated in place
 *   answer_len_dev device int32 [n_questions], in/out: tokens of each cached answer
 *                  (new = old - m_k + tokens of the selected response)
 *   question_dev   device int32 [n_groups] or NULL: pool row of batch group k (as in rpo_cut_pack);
 *                  every other array below is in batch order
 *   m_dev          device int32 [n_groups]: tokens cut from each answer in this step
 *   tokens_dev     device int32 [n_groups*G, tok_stride]: sampled tokens, row r = k*G + i
 *   lengths_dev    device int32 [n_groups*G] or NULL: tokens each rollout generated (rpo_sample's
 *                  lengths; NULL = m_k, the fixed-length case)
 *   rewards_dev    device fp32 [n_groups, G]; u_dev device fp32 [n_groups] in [0, 1);
 *   g_prime_dev    device int32 [n_groups] in [0, G)
 *   chosen_out_dev device int32 [n_groups] or NULL: the selected index
 * A question whose cut or new length does not fit its pool row (or whose g' is out of range) is
 * left unchanged and reports -1.  Errors: RPO_EINVAL (NULL, sizes, eps outside [0, 1]). */
int rpo_cache_update(int32_t *pool_dev, int64_t pool_stride, int32_t *answer_len_dev,
                     const int32_t *question_dev, const int32_t *m_dev, const int32_t *tokens_dev, int64_t tok_stride, const int32_t *lengths_dev,
                     const float *rewards_dev, const float *u_dev, const int32_t *g_prime_dev, int32_t n_groups,
                     int32_t G, float eps, int32_t *chosen_out_dev, void *stream);

/* Thread-local message of the last failing call in this thread ("" if none). */
const char *rpo_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RPO_H */
