// Temperature sampling, log-sum-exp gather and group-relative advantages.
//
// This translation unit is compiled with -ffp-contract=off: the sampler's
// arithmetic is a bit-exact contract (see rpo_sample in rpo.h), every fp32
// multiply and add below must round on its own.
#include "kernels.hpp"

namespace rpo {

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): 10 rounds, multipliers 0xD2511F53 /
// 0xCD9E8D57, Weyl key increments 0x9E3779B9 / 0xBB67AE85.
// ---------------------------------------------------------------------------
__device__ inline uint64_t philox_u64(uint64_t seed, uint64_t seq, uint32_t step) {
    uint32_t c0 = step, c1 = (uint32_t)seq, c2 = (uint32_t)(seq >> 32), c3 = 0u;
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        if (r) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0;
        c1 = n1;
        c2 = n2;
        c3 = n3;
    }
    return ((uint64_t)c1 << 32) | c0;
}

// q = floor(2^x * 2^40) through the fixed polynomial; x = ((z - zmax) * inv_t) * log2(e).
__device__ inline uint64_t weight_u64(float z, float zmax, float inv_t) {
    float x = __fsub_rn(z, zmax);
    x = __fmul_rn(x, inv_t);
    x = __fmul_rn(x, 0x1.715476p+0f);
    if (!(x >= -41.0f)) return 0ull;  // also catches NaN
    const float n = __builtin_rintf(x);
    const float f = __fsub_rn(x, n);
    float p = 0x1.ffcbfcp-17f;
    p = __fadd_rn(__fmul_rn(p, f), 0x1.430912p-13f);
    p = __fadd_rn(__fmul_rn(p, f), 0x1.5d87fep-10f);
    p = __fadd_rn(__fmul_rn(p, f), 0x1.3b2ab6p-7f);
    p = __fadd_rn(__fmul_rn(p, f), 0x1.c6b08ep-5f);
    p = __fadd_rn(__fmul_rn(p, f), 0x1.ebfbe0p-3f);
    p = __fadd_rn(__fmul_rn(p, f), 0x1.62e430p-1f);
    p = __fadd_rn(__fmul_rn(p, f), 1.0f);
    // p = m * 2^(E - 23) with a 24-bit integer m and E in {-1, 0}; floor(p * 2^(n + 40)) is a shift
    // of m by E - 23 + n + 40 in [-25, 17] (exact integer arithmetic, truncation == floor).
    const uint32_t bits = __float_as_uint(p);
    const uint32_t m = (bits & 0x7fffffu) | 0x800000u;
    const int sh = (int)(bits >> 23) - 127 - 23 + (int)n + 40;
    return sh >= 0 ? ((uint64_t)m << sh) : (uint64_t)(m >> (-sh));
}

// Sum over the wave of values < 2^45: two 32-bit sums (low 22 bits, high bits) so each
// cross-lane step moves one register.
__device__ inline uint64_t wave_sum_u45(uint64_t v) {
    uint32_t lo = (uint32_t)v & 0x3fffffu, hi = (uint32_t)(v >> 22);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        lo += __shfl_xor(lo, o, kWave);
        hi += __shfl_xor(hi, o, kWave);
    }
    return ((uint64_t)hi << 22) + lo;
}
__device__ inline uint64_t wave_sum_u64(uint64_t v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)v, o, kWave);
        const uint32_t hi = __shfl_xor((uint32_t)(v >> 32), o, kWave);
        v += ((uint64_t)hi << 32) | lo;
    }
    return v;
}

// Four consecutive logits starting at i (values beyond V read as -inf); one 16-byte load when
// the row allows it.
__device__ inline float4 load4(const float* z, int i, int V, bool vec) {
    if (vec && i + 3 < V) return *(const float4*)(z + i);
    float4 r;
    r.x = i < V ? z[i] : -INFINITY;
    r.y = i + 1 < V ? z[i + 1] : -INFINITY;
    r.z = i + 2 < V ? z[i + 2] : -INFINITY;
    r.w = i + 3 < V ? z[i + 3] : -INFINITY;
    return r;
}

// One workgroup (NW waves) per output row.  The row is cut into segments of 1024 logits =
// 4 sub-blocks of 256 (4 per lane); wave w owns segments w, w + NW, ...  Integer sums make
// the result independent of this decomposition.
constexpr int kSubLen = 256;
constexpr int kSegLen = 1024;
constexpr int kMaxSeg = 256;  // vocab <= 262144

// NW waves per row: few rows need many waves each to keep the vector ALUs busy.
template <int NW>
__global__ __launch_bounds__(NW * 64) void sample_kernel(SampleArgs a) {
    __shared__ uint64_t seg_sum[kMaxSeg];
    __shared__ float red[NW];
    __shared__ int pick_seg;
    __shared__ uint64_t pick_rem, row_total;
    const int r = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (a.active && !a.active[r]) {  // finished rollout: no draw, the output is padding
        if (tid == 0) {
            a.tokens_out[r] = a.eos_id >= 0 ? a.eos_id : 0;
            if (a.logprob_out) a.logprob_out[r] = 0.f;
        }
        return;
    }
    const int src = a.row_map ? a.row_map[r] : r;
    const float* z = a.logits + (int64_t)src * a.row_stride;
    const int V = a.vocab;
    const int n_seg = (V + kSegLen - 1) / kSegLen;
    const bool vec = ((uintptr_t)z % 16) == 0;

    float zmax = -INFINITY;
    if (a.row_max) {  // the caller (the LM-head epilogue) already knows the row's maximum
        zmax = a.row_max[src];
    } else {
        for (int i = tid * 4; i < V; i += NW * 256) {
            const float4 v = load4(z, i, V, vec);
            zmax = fmaxf(fmaxf(zmax, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
        }
        zmax = wave_max(zmax);
        if (lane == 0) red[wave] = zmax;
        __syncthreads();
        zmax = red[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) zmax = fmaxf(zmax, red[w]);
    }

    // The logits of the wave's next segment are loaded while the weights of the current one are
    // computed (-inf beyond the row: weight 0).
    float4 cur[4], nxt[4];
#pragma unroll
    for (int sb = 0; sb < 4; ++sb) cur[sb] = load4(z, wave * kSegLen + sb * kSubLen + lane * 4, V, vec);
    for (int sg = wave; sg < n_seg; sg += NW) {
        const bool more = sg + NW < n_seg;  // wave-uniform
        if (more) {
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) nxt[sb] = load4(z, (sg + NW) * kSegLen + sb * kSubLen + lane * 4, V, vec);
        }
        uint64_t q = 0;  // < 16 * 2^41
#pragma unroll
        for (int sb = 0; sb < 4; ++sb) {
            const float4 v = cur[sb];
            q += weight_u64(v.x, zmax, a.inv_t) + weight_u64(v.y, zmax, a.inv_t) +
                 weight_u64(v.z, zmax, a.inv_t) + weight_u64(v.w, zmax, a.inv_t);
        }
        q = wave_sum_u45(q);
        if (lane == 0) seg_sum[sg] = q;
        if (more) {
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) cur[sb] = nxt[sb];
        }
    }
    __syncthreads();

    if (wave == 0) {
        // total, threshold, and the segment the threshold falls into
        uint64_t loc = 0;
        for (int sg = lane; sg < n_seg; sg += 64) loc += seg_sum[sg];
        const uint64_t total = wave_sum_u64(loc);
        const uint64_t u = philox_u64(a.seed, a.seq_id[r], a.step);
        const uint64_t t = __umul64hi(u, total);
        if (lane == 0) {
            uint64_t run = 0;
            int sg = 0;
            for (; sg < n_seg - 1; ++sg) {
                if (run + seg_sum[sg] > t) break;
                run += seg_sum[sg];
            }
            pick_seg = sg;
            pick_rem = t - run;  // < seg_sum[sg]
            row_total = total;
        }
    }
    __syncthreads();
    if (wave == 0) {
        uint64_t rem = pick_rem;
        // walk the 4 sub-blocks of the chosen segment in vocabulary order
        for (int sb = 0; sb < 4; ++sb) {
            const int i0 = pick_seg * kSegLen + sb * kSubLen + lane * 4;
            const float4 v = load4(z, i0, V, vec);
            uint64_t q[4];
            q[0] = weight_u64(v.x, zmax, a.inv_t);
            q[1] = weight_u64(v.y, zmax, a.inv_t);
            q[2] = weight_u64(v.z, zmax, a.inv_t);
            q[3] = weight_u64(v.w, zmax, a.inv_t);
            const uint64_t mine = q[0] + q[1] + q[2] + q[3];
            uint64_t incl = mine;  // inclusive prefix over lanes
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t lo = __shfl_up((uint32_t)incl, o, kWave);
                const uint32_t hi = __shfl_up((uint32_t)(incl >> 32), o, kWave);
                if (lane >= o) incl += ((uint64_t)hi << 32) | lo;
            }
            const uint32_t blo = __shfl((uint32_t)incl, 63, kWave), bhi = __shfl((uint32_t)(incl >> 32), 63, kWave);
            const uint64_t block_total = ((uint64_t)bhi << 32) | blo;
            if (rem >= block_total) {  // uniform across the wave
                rem -= block_total;
                continue;
            }
            const uint64_t excl = incl - mine;
            if (excl <= rem && rem < incl) {  // exactly one lane
                uint64_t run = excl;
                int tok = i0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (run + q[e] > rem) {
                        tok = i0 + e;
                        break;
                    }
                    run += q[e];
                }
                a.tokens_out[r] = tok;
                if (a.lengths) a.lengths[r] += 1;
                if (a.active && a.eos_id >= 0 && tok == a.eos_id) a.active[r] = 0;
                if (a.logprob_out) {
                    const float x = ((z[tok] - zmax) * a.inv_t);
                    a.logprob_out[r] = x - (float)(log((double)row_total) - 40.0 * 0.6931471805599453);
                }
            }
            break;
        }
    }
}

hipError_t launch_sample(const SampleArgs& a, hipStream_t s) {
    if (a.n_out_rows <= 0) return hipSuccess;
    if (a.vocab > kSegLen * kMaxSeg) return hipErrorInvalidValue;
    // up to ~4 rows per CU: 16 waves per row (the sweep is ALU work, 27 operations per logit)
    if (a.n_out_rows <= 1024)
        sample_kernel<16><<<a.n_out_rows, 1024, 0, s>>>(a);
    else
        sample_kernel<4><<<a.n_out_rows, 256, 0, s>>>(a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// out[r] = z[target] * inv_t - logsumexp(z * inv_t): one workgroup per row.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lse_gather_kernel(const float* __restrict__ logits,
                                                         int64_t row_stride, int vocab,
                                                         const int32_t* __restrict__ target, float inv_t,
                                                         float* __restrict__ out) {
    __shared__ float red[4];
    __shared__ float red2[4];
    const int r = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* z = logits + (int64_t)r * row_stride;
    const bool vec = ((uintptr_t)z % 16) == 0;
    float mx = -INFINITY;
    for (int i = tid * 4; i < vocab; i += 1024) {
        const float4 v = load4(z, i, vocab, vec);
        mx = fmaxf(fmaxf(mx, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
    }
    mx = wave_max(mx);
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float k2 = inv_t * 1.4426950408889634f;  // exp(y) = 2^(y * log2 e)
    float sum = 0.f;
    for (int i = tid * 4; i < vocab; i += 1024) {
        const float4 v = load4(z, i, vocab, vec);  // -inf padding contributes 2^-inf = 0
        sum += (exp2f((v.x - mx) * k2) + exp2f((v.y - mx) * k2)) + (exp2f((v.z - mx) * k2) + exp2f((v.w - mx) * k2));
    }
    sum = wave_sum(sum);
    if (lane == 0) red2[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        const float tot = (red2[0] + red2[1]) + (red2[2] + red2[3]);
        const int t = target[r];
        const float zt = (t >= 0 && t < vocab) ? z[t] : NAN;
        out[r] = (zt - mx) * inv_t - logf(tot);
    }
}

// One workgroup per row: the maximum over its block maxima / over the row itself.
__global__ __launch_bounds__(256) void row_max_blocks_kernel(const float* __restrict__ part, int blocks,
                                                             float* __restrict__ out) {
    __shared__ float red[4];
    const int r = blockIdx.x, tid = threadIdx.x;
    float mx = -INFINITY;
    for (int b = tid; b < blocks; b += 256) mx = fmaxf(mx, part[(int64_t)r * blocks + b]);
    mx = wave_max(mx);
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    if (tid == 0) out[r] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__global__ __launch_bounds__(256) void row_max_kernel(const float* __restrict__ logits, int64_t row_stride, int vocab,
                                                      float* __restrict__ out) {
    __shared__ float red[4];
    const int r = blockIdx.x, tid = threadIdx.x;
    const float* z = logits + (int64_t)r * row_stride;
    const bool vec = ((uintptr_t)z % 16) == 0;
    float mx = -INFINITY;
    for (int i = tid * 4; i < vocab; i += 1024) {
        const float4 v = load4(z, i, vocab, vec);  // -inf beyond the row
        mx = fmaxf(fmaxf(mx, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
    }
    mx = wave_max(mx);
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    if (tid == 0) out[r] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

hipError_t launch_row_max_blocks(const float* part, int blocks, float* out, int rows, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    row_max_blocks_kernel<<<rows, 256, 0, s>>>(part, blocks, out);
    return hipGetLastError();
}

hipError_t launch_row_max(const float* logits, int64_t row_stride, int vocab, float* out, int rows, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    row_max_kernel<<<rows, 256, 0, s>>>(logits, row_stride, vocab, out);
    return hipGetLastError();
}

// One wave per row: merge the (max, sum) pieces of the fused LM-head epilogue.
__global__ __launch_bounds__(64) void lse_combine_kernel(const float* __restrict__ part, int blocks,
                                                         const float* __restrict__ target_logit,
                                                         const int32_t* __restrict__ target, int vocab, float inv_t,
                                                         float* __restrict__ out) {
    const int r = blockIdx.x, lane = threadIdx.x;
    const float* p = part + (int64_t)r * blocks * 2;
    float mx = -INFINITY;
    for (int b = lane; b < blocks; b += 64) mx = fmaxf(mx, p[2 * b]);
    mx = wave_max(mx);
    const float k2 = inv_t * 1.4426950408889634f;
    float sum = 0.f;
    for (int b = lane; b < blocks; b += 64) {
        const float m = p[2 * b];
        if (m != -INFINITY) sum += p[2 * b + 1] * exp2f((m - mx) * k2);
    }
    sum = wave_sum(sum);
    if (lane == 0) {
        const int t = target[r];
        const float zt = (t >= 0 && t < vocab) ? target_logit[r] : NAN;  // as launch_lse_gather
        out[r] = (zt - mx) * inv_t - logf(sum);
    }
}

hipError_t launch_lse_combine(const float* part, int blocks, const float* target_logit, const int32_t* target,
                              int vocab, float inv_t, float* out, int rows, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    lse_combine_kernel<<<rows, 64, 0, s>>>(part, blocks, target_logit, target, vocab, inv_t, out);
    return hipGetLastError();
}

hipError_t launch_lse_gather(const float* logits, int64_t row_stride, int vocab, const int32_t* target,
                             float inv_t, float* out, int rows, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    lse_gather_kernel<<<rows, 256, 0, s>>>(logits, row_stride, vocab, target, inv_t, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Eq. 7 of the paper: A_i = (R_i - mean) / (std + eps); one thread per group,
// left-to-right fp64 sums (IEEE add / mul / div / sqrt: same bits as a CPU loop).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void advantages_kernel(const float* __restrict__ rewards, int n_groups,
                                                        int G, int ddof, float eps,
                                                        float* __restrict__ adv) {
    const int k = blockIdx.x * 64 + threadIdx.x;
    if (k >= n_groups) return;
    const float* r = rewards + (int64_t)k * G;
    float* o = adv + (int64_t)k * G;
    double s = 0.0;
    for (int i = 0; i < G; ++i) s += (double)r[i];
    const double mu = s / (double)G;
    double ss = 0.0;
    for (int i = 0; i < G; ++i) {
        const double d = (double)r[i] - mu;
        ss += d * d;
    }
    const double sigma = __dsqrt_rn(ss / (double)(G - ddof));
    const double e = (double)eps;
    if (sigma == 0.0 && e == 0.0) {
        for (int i = 0; i < G; ++i) o[i] = 0.0f;
        return;
    }
    const double den = sigma + e;
    for (int i = 0; i < G; ++i) o[i] = (float)(((double)r[i] - mu) / den);
}

// Eq. 11 of the paper: R = clip(r / (1 + exp(-alpha (l_ref - len))), lo, hi) for r > 0, else 0;
// l_ref = mean response length of the group.  One thread per group, fp64.
__global__ __launch_bounds__(64) void shape_rewards_kernel(const float* __restrict__ rewards,
                                                           const int32_t* __restrict__ lengths, int n_groups,
                                                           int G, float alpha, float lo, float hi,
                                                           float* __restrict__ out) {
    const int k = blockIdx.x * 64 + threadIdx.x;
    if (k >= n_groups) return;
    const float* r = rewards + (int64_t)k * G;
    const int32_t* ln = lengths + (int64_t)k * G;
    float* o = out + (int64_t)k * G;
    double s = 0.0;
    for (int i = 0; i < G; ++i) s += (double)ln[i];
    const double l_ref = s / (double)G;
    for (int i = 0; i < G; ++i) {
        const double raw = (double)r[i];
        double v = 0.0;
        if (raw > 0.0) {
            const double w = 1.0 / (1.0 + exp(-(double)alpha * (l_ref - (double)ln[i])));
            v = fmin(fmax(raw * w, (double)lo), (double)hi);
        }
        o[i] = (float)v;
    }
}

// Eq. 5-7 of the paper, forward value.  One thread per rollout walks its tokens (fp64):
// surrogate l = min(r A, clip(r, 1 - eps, 1 + eps) A), r = exp(lp_new - lp_old); the rollout's
// share is (sum l - beta * sum (lp_new - lp_ref)) / |o|.  A second kernel averages each group.
__global__ __launch_bounds__(64) void objective_rollout_kernel(const float* __restrict__ lp_new,
                                                               const float* __restrict__ lp_old,
                                                               const float* __restrict__ lp_ref,
                                                               const int32_t* __restrict__ cu,
                                                               const float* __restrict__ adv, int n_rollouts,
                                                               float eps_clip, float beta,
                                                               float* __restrict__ tok_out,
                                                               double* __restrict__ per_rollout) {
    const int r = blockIdx.x * 64 + threadIdx.x;
    if (r >= n_rollouts) return;
    const int lo = cu[r], hi = cu[r + 1];
    const double a = (double)adv[r], e = (double)eps_clip, b = (double)beta;
    double s = 0.0, kl = 0.0;
    for (int t = lo; t < hi; ++t) {
        const double ln = (double)lp_new[t];
        const double ratio = exp(ln - (double)lp_old[t]);
        const double rc = fmin(fmax(ratio, 1.0 - e), 1.0 + e);
        const double l = fmin(ratio * a, rc * a);
        if (tok_out) tok_out[t] = (float)l;
        s += l;
        if (lp_ref) kl += ln - (double)lp_ref[t];
    }
    per_rollout[r] = hi > lo ? (s - b * kl) / (double)(hi - lo) : 0.0;
}

__global__ __launch_bounds__(64) void objective_group_kernel(const double* __restrict__ per_rollout, int n_groups,
                                                             int G, float* __restrict__ j_out) {
    const int k = blockIdx.x * 64 + threadIdx.x;
    if (k >= n_groups) return;
    double acc = 0.0;
    for (int i = 0; i < G; ++i) acc += per_rollout[(int64_t)k * G + i];
    j_out[k] = (float)(acc / (double)G);
}

hipError_t launch_objective(const float* lp_new, const float* lp_old, const float* lp_ref, const int32_t* cu,
                            const float* adv, int n_groups, int G, float eps_clip, float beta, float* tok_out,
                            double* per_rollout, float* j_out, hipStream_t s) {
    const int n = n_groups * G;
    if (n <= 0) return hipSuccess;
    objective_rollout_kernel<<<ceil_div(n, 64), 64, 0, s>>>(lp_new, lp_old, lp_ref, cu, adv, n, eps_clip, beta,
                                                           tok_out, per_rollout);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    objective_group_kernel<<<ceil_div(n_groups, 64), 64, 0, s>>>(per_rollout, n_groups, G, j_out);
    return hipGetLastError();
}

hipError_t launch_shape_rewards(const float* rewards, const int32_t* lengths, int n_groups, int G, float alpha,
                                float lo, float hi, float* out, hipStream_t s) {
    if (n_groups <= 0) return hipSuccess;
    shape_rewards_kernel<<<ceil_div(n_groups, 64), 64, 0, s>>>(rewards, lengths, n_groups, G, alpha, lo, hi, out);
    return hipGetLastError();
}

hipError_t launch_advantages(const float* rewards, int n_groups, int G, int ddof, float eps, float* adv,
                             hipStream_t s) {
    if (n_groups <= 0) return hipSuccess;
    advantages_kernel<<<ceil_div(n_groups, 64), 64, 0, s>>>(rewards, n_groups, G, ddof, eps, adv);
    return hipGetLastError();
}

}  // namespace rpo
