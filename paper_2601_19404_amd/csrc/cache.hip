// Device side of the experience cache (RPO Sec. 3.1-3.3, Algorithm 1): the cached answers live in
// HBM as an int32 pool [n_groups, stride]; the cut of Eq. 3 packs prompt || kept answer prefix for
// the prefill, and the epsilon-greedy rule around Eq. 10 writes the selected response's suffix back
// in place.  Integer work only.
#include "kernels.hpp"

namespace rpo {

// One workgroup per batch group k (question row qi = question ? question[k] : k):
// out[cu[k] + t] = t < P ? prompt[qi][t] : answer[qi][t - P].
__global__ __launch_bounds__(256) void cut_pack_kernel(const int32_t* __restrict__ prompts, int64_t prompt_stride,
                                                       const int32_t* __restrict__ prompt_len,
                                                       const int32_t* __restrict__ pool, int64_t pool_stride,
                                                       const int32_t* __restrict__ question,
                                                       const int32_t* __restrict__ cu_len,
                                                       int32_t* __restrict__ out) {
    const int k = blockIdx.x;
    const int64_t qi = question ? question[k] : k;
    const int begin = cu_len[k], len = cu_len[k + 1] - begin, P = prompt_len[qi];
    const int32_t* q = prompts + qi * prompt_stride;
    const int32_t* a = pool + qi * pool_stride;
    for (int t = threadIdx.x; t < len; t += 256) out[begin + t] = t < P ? q[t] : a[t - P];
}

hipError_t launch_cut_pack(const int32_t* prompts, int64_t prompt_stride, const int32_t* prompt_len,
                           const int32_t* pool, int64_t pool_stride, const int32_t* question,
                           const int32_t* cu_len, int n_groups, int32_t* out, hipStream_t s) {
    if (n_groups <= 0) return hipSuccess;
    cut_pack_kernel<<<n_groups, 256, 0, s>>>(prompts, prompt_stride, prompt_len, pool, pool_stride, question, cu_len,
                                             out);
    return hipGetLastError();
}

// One workgroup per batch group k (question row qi as above).  Selection: u_k <= eps -> the response with the highest reward
// (lowest index on ties), otherwise response g'_k.  The new answer is the kept prefix
// a_k[0 : len_k - m_k] followed by the tokens the selected rollout generated.
__global__ __launch_bounds__(256) void cache_update_kernel(int32_t* __restrict__ pool, int64_t pool_stride,
                                                           int32_t* __restrict__ answer_len,
                                                           const int32_t* __restrict__ question,
                                                           const int32_t* __restrict__ m,
                                                           const int32_t* __restrict__ tokens, int64_t tok_stride,
                                                           const int32_t* __restrict__ lengths,
                                                           const float* __restrict__ rewards,
                                                           const float* __restrict__ u,
                                                           const int32_t* __restrict__ g_prime, int G, float eps,
                                                           int32_t* __restrict__ chosen_out) {
    const int k = blockIdx.x;
    int pick;
    if (u[k] <= eps) {
        pick = 0;
        float best = rewards[(int64_t)k * G];
        for (int i = 1; i < G; ++i) {
            const float r = rewards[(int64_t)k * G + i];
            if (r > best) {
                best = r;
                pick = i;
            }
        }
    } else {
        pick = g_prime[k];
    }
    const int64_t qi = question ? question[k] : k;
    const int mk = m[k], old_len = answer_len[qi];
    const int keep = old_len - mk;
    const int64_t row = (int64_t)k * G + pick;
    const bool pick_ok = pick >= 0 && pick < G;
    const int n_new = pick_ok ? (lengths ? lengths[row] : mk) : 0;
    // an entry whose cut or new length does not fit is left as it is and reports -1
    const bool ok = pick_ok && mk >= 0 && keep >= 0 && n_new >= 0 && n_new <= tok_stride &&
                    (int64_t)keep + n_new <= pool_stride;
    if (ok) {
        const int32_t* src = tokens + row * tok_stride;
        int32_t* dst = pool + qi * pool_stride + keep;
        for (int t = threadIdx.x; t < n_new; t += 256) dst[t] = src[t];
    }
    if (threadIdx.x == 0) {
        if (ok) answer_len[qi] = keep + n_new;
        if (chosen_out) chosen_out[k] = ok ? pick : -1;
    }
}

hipError_t launch_cache_update(int32_t* pool, int64_t pool_stride, int32_t* answer_len, const int32_t* question,
                               const int32_t* m,
                               const int32_t* tokens, int64_t tok_stride, const int32_t* lengths,
                               const float* rewards, const float* u, const int32_t* g_prime, int n_groups, int G,
                               float eps, int32_t* chosen_out, hipStream_t s) {
    if (n_groups <= 0) return hipSuccess;
    cache_update_kernel<<<n_groups, 256, 0, s>>>(pool, pool_stride, answer_len, question, m, tokens, tok_stride, lengths,
                                                  rewards, u, g_prime, G, eps, chosen_out);
    return hipGetLastError();
}

}  // namespace rpo
