// Shared host/device helpers for the RPO rollout kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rpo {

constexpr int kWave = 64;  // CDNA wavefront width

// 16-byte register value for staging global -> LDS copies (a native vector: stays in VGPRs).
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// bfloat16 as raw bits: conversions are explicit so rounding is always RNE.
struct bf16 {
    uint16_t bits;
};

__host__ __device__ inline float bf16_to_f32(bf16 v) {
    union {
        uint32_t u;
        float f;
    } c;
    c.u = static_cast<uint32_t>(v.bits) << 16;
    return c.f;
}

__host__ __device__ inline bf16 f32_to_bf16(float f) {
#if defined(__HIP_DEVICE_COMPILE__)
    // the hardware conversion (round to nearest even, quiet NaN)
    const __bf16 h = (__bf16)f;
    bf16 r;
    r.bits = __builtin_bit_cast(uint16_t, h);
    return r;
#else
    union {
        uint32_t u;
        float f;
    } c;
    c.f = f;
    uint32_t u = c.u;
    bf16 r;
    if ((u & 0x7fffffffu) > 0x7f800000u) {  // NaN stays NaN
        r.bits = static_cast<uint16_t>((u >> 16) | 0x40u);
        return r;
    }
    u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even
    r.bits = static_cast<uint16_t>(u >> 16);
    return r;
#endif
}

template <typename T>
__device__ inline float to_f32(T v);
template <>
__device__ inline float to_f32<float>(float v) {
    return v;
}
template <>
__device__ inline float to_f32<bf16>(bf16 v) {
    return bf16_to_f32(v);
}

template <typename T>
__device__ inline T from_f32(float v);
template <>
__device__ inline float from_f32<float>(float v) {
    return v;
}
template <>
__device__ inline bf16 from_f32<bf16>(float v) {
    return f32_to_bf16(v);
}

// Wave-wide reductions through cross-lane shuffles (64 lanes).
__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------------------
// Paged KV cache geometry.
//
// pool[layer][page][K|V][kv_head][...]: for K the inner block is
// [page_tokens][head_dim] (a token's key is contiguous), for V it is
// [page_tokens / 8][head_dim][8] (transposed in groups of eight tokens: the P*V matrix product
// wants eight consecutive tokens of one channel per lane, exactly one 16-byte unit, and a
// token's head_dim values land 16 bytes apart -- 16 cache lines per token instead of 128).
// ---------------------------------------------------------------------------
struct KvGeom {
    int n_kv_heads, head_dim, page_tokens;
    int64_t n_pages;  // pages per layer
    __host__ __device__ int64_t head_block() const { return (int64_t)page_tokens * head_dim; }
    __host__ __device__ int64_t page_stride() const { return 2 * n_kv_heads * head_block(); }
    __host__ __device__ int64_t layer_stride() const { return n_pages * page_stride(); }
    __host__ __device__ int64_t k_block(int layer, int64_t page, int h) const {
        return layer * layer_stride() + page * page_stride() + (int64_t)h * head_block();
    }
    __host__ __device__ int64_t v_block(int layer, int64_t page, int h) const {
        return layer * layer_stride() + page * page_stride() + (int64_t)(n_kv_heads + h) * head_block();
    }
    // element (token slot, channel d) inside a V block; page_tokens is a multiple of 8
    __host__ __device__ int64_t v_elem(int slot, int d) const {
        return ((int64_t)(slot >> 3) * head_dim + d) * 8 + (slot & 7);
    }
};

}  // namespace rpo
