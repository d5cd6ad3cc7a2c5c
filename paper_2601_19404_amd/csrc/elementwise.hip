// Bandwidth-bound row kernels of the decoder: embedding gather, RMSNorm, rotary
// embedding + KV page write, SwiGLU, and the page copy of the KV fork.
#include "kernels.hpp"

namespace rpo {

// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const int32_t* __restrict__ tokens,
                                                    const int32_t* __restrict__ tok_index,
                                                    const T* __restrict__ embed, int vocab, int d,
                                                    float* __restrict__ x) {
    const int r = blockIdx.x;
    const int idx = tok_index ? tok_index[r] : r;
    const int tok = idx >= 0 ? tokens[idx] : -1;
    const bool ok = tok >= 0 && tok < vocab;
    const T* src = embed + (int64_t)(ok ? tok : 0) * d;
    float* dst = x + (int64_t)r * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) dst[c] = ok ? to_f32<T>(src[c]) : 0.0f;
}

hipError_t launch_embed(const int32_t* tokens, const int32_t* tok_index, const void* embed, int dtype,
                        int vocab, int d, float* x, int rows, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    if (dtype == kF32)
        embed_kernel<float><<<rows, 256, 0, s>>>(tokens, tok_index, (const float*)embed, vocab, d, x);
    else
        embed_kernel<bf16><<<rows, 256, 0, s>>>(tokens, tok_index, (const bf16*)embed, vocab, d, x);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// One workgroup per row.  Mean of squares in fp32 (wave shuffles, then LDS across
// the four waves).
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x,
                                                      const int32_t* __restrict__ row_idx,
                                                      const T* __restrict__ gain, int d, float eps,
                                                      T* __restrict__ h) {
    __shared__ float part[4];
    const int r = blockIdx.x;
    const int64_t src = row_idx ? row_idx[r] : r;
    const float* xr = x + src * d;
    float ss = 0.0f;
    for (int c = threadIdx.x; c < d; c += 256) {
        const float v = xr[c];
        ss += v * v;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = (part[0] + part[1]) + (part[2] + part[3]);
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    T* hr = h + (int64_t)r * d;
    for (int c = threadIdx.x; c < d; c += 256) hr[c] = from_f32<T>(xr[c] * inv * to_f32<T>(gain[c]));
}

// One wave per row, the row held in registers (NV float4 per lane: d <= 256 NV, d a multiple of
// 4): x is read once with 16-byte loads, h leaves in 8- / 16-byte stores, no LDS.
template <typename T, int NV>
__global__ __launch_bounds__(256) void rmsnorm_wave_kernel(const float* __restrict__ x,
                                                           const int32_t* __restrict__ row_idx,
                                                           const T* __restrict__ gain, int d, float eps,
                                                           T* __restrict__ h, int rows) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int64_t src = row_idx ? row_idx[r] : r;
    const float4* xr = (const float4*)(x + src * d);
    const int nv = d >> 2;
    float4 v[NV];
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = i * 64 + lane;
        v[i] = c < nv ? xr[c] : float4{0.f, 0.f, 0.f, 0.f};
        ss += (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
    }
    ss = wave_sum(ss);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    T* hr = h + (int64_t)r * d;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = i * 64 + lane;
        if (c >= nv) continue;
        T g4[4], o4[4];
        if constexpr (sizeof(T) == 2)
            *(uint2*)g4 = *(const uint2*)(gain + 4 * c);
        else
            *(float4*)g4 = *(const float4*)(gain + 4 * c);
        o4[0] = from_f32<T>(v[i].x * inv * to_f32<T>(g4[0]));
        o4[1] = from_f32<T>(v[i].y * inv * to_f32<T>(g4[1]));
        o4[2] = from_f32<T>(v[i].z * inv * to_f32<T>(g4[2]));
        o4[3] = from_f32<T>(v[i].w * inv * to_f32<T>(g4[3]));
        if constexpr (sizeof(T) == 2)
            *(uint2*)(hr + 4 * c) = *(const uint2*)o4;
        else
            *(float4*)(hr + 4 * c) = *(const float4*)o4;
    }
}

template <typename T>
static bool launch_rmsnorm_wave(const float* x, const int32_t* row_idx, const T* gain, int d, float eps, T* h,
                                int rows, hipStream_t s) {
    if (d % 4 != 0 || d > 4096 || (uintptr_t)x % 16 != 0 || (uintptr_t)gain % 16 != 0 || (uintptr_t)h % 16 != 0)
        return false;
    const int grid = ceil_div(rows, 4);
    if (d <= 1536)
        rmsnorm_wave_kernel<T, 6><<<grid, 256, 0, s>>>(x, row_idx, gain, d, eps, h, rows);
    else
        rmsnorm_wave_kernel<T, 16><<<grid, 256, 0, s>>>(x, row_idx, gain, d, eps, h, rows);
    return true;
}

hipError_t launch_rmsnorm(const float* x, const int32_t* row_idx, const void* gain, int dtype, int d,
                          float eps, void* h, int rows, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    if (dtype == kF32 ? launch_rmsnorm_wave<float>(x, row_idx, (const float*)gain, d, eps, (float*)h, rows, s)
                      : launch_rmsnorm_wave<bf16>(x, row_idx, (const bf16*)gain, d, eps, (bf16*)h, rows, s))
        return hipGetLastError();
    if (dtype == kF32)
        rmsnorm_kernel<float><<<rows, 256, 0, s>>>(x, row_idx, (const float*)gain, d, eps, (float*)h);
    else
        rmsnorm_kernel<bf16><<<rows, 256, 0, s>>>(x, row_idx, (const bf16*)gain, d, eps, (bf16*)h);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void swiglu_kernel(const T* __restrict__ gu, int F,
                                                     T* __restrict__ act) {
    const int r = blockIdx.x;
    const int j = blockIdx.y * 256 + threadIdx.x;
    if (j >= F) return;
    const T* row = gu + (int64_t)r * 2 * F;
    const float g = to_f32<T>(row[j]);
    const float u = to_f32<T>(row[F + j]);
    const float sg = g / (1.0f + expf(-g));
    act[(int64_t)r * F + j] = from_f32<T>(sg * u);
}

hipError_t launch_swiglu(const void* gu, int dtype, int F, void* act, int rows, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    dim3 grid(rows, ceil_div(F, 256));
    if (dtype == kF32)
        swiglu_kernel<float><<<grid, 256, 0, s>>>((const float*)gu, F, (float*)act);
    else
        swiglu_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)gu, F, (bf16*)act);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_rows_kernel(const float* __restrict__ src,
                                                          const int32_t* __restrict__ row_idx, int d,
                                                          float* __restrict__ dst) {
    const int r = blockIdx.x;
    const float* s = src + (int64_t)row_idx[r] * d;
    float* o = dst + (int64_t)r * d;
    for (int c = threadIdx.x; c < d; c += 256) o[c] = s[c];
}

hipError_t launch_gather_rows(const float* src, const int32_t* row_idx, int d, float* dst, int rows,
                              hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    gather_rows_kernel<<<rows, 256, 0, s>>>(src, row_idx, d, dst);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// One workgroup per token row.  Work items: (Hq + Hkv) * dh/2 rotation pairs, then
// Hkv * dh value elements.  Rotation in fp32 from the precomputed (cos, sin) table.
template <typename T>
__global__ __launch_bounds__(256) void rope_kv_kernel(RopeKvArgs a) {
    const int r = blockIdx.x;
    if (a.active && !a.active[r]) return;
    const int seq = a.row_seq ? a.row_seq[r] : r;
    if (seq < 0) return;
    const SeqDesc sd = a.seqs[seq];
    const int pos = sd.pos0 + (a.single_row ? 0 : r - sd.row_start) + a.pos_add;
    const int pt = a.geom.page_tokens;
    const int64_t page = a.tables[sd.table_off + pos / pt];
    const int slot = pos % pt;
    const int dh = a.dh, half = dh / 2;
    const int width = (a.Hq + 2 * a.Hkv) * dh;
    T* row = (T*)a.qkv + (int64_t)r * width;
    T* pool = (T*)a.kv_pool;
    const float* cs = a.rope + (int64_t)pos * half * 2;

    const int n_rot = (a.Hq + a.Hkv) * half;
    for (int w = threadIdx.x; w < n_rot; w += 256) {
        const int head = w / half, i = w % half;
        const float c = cs[2 * i], s = cs[2 * i + 1];
        T* hp = row + (int64_t)head * dh;  // q heads first, k heads follow directly
        const float x1 = to_f32<T>(hp[i]);
        const float x2 = to_f32<T>(hp[i + half]);
        const T y1 = from_f32<T>(x1 * c - x2 * s);
        const T y2 = from_f32<T>(x2 * c + x1 * s);
        if (head < a.Hq) {
            hp[i] = y1;
            hp[i + half] = y2;
        } else {
            const int kh = head - a.Hq;
            T* kdst = pool + a.geom.k_block(a.layer, page, kh) + (int64_t)slot * dh;
            kdst[i] = y1;
            kdst[i + half] = y2;
        }
    }
    const T* vsrc = row + (int64_t)(a.Hq + a.Hkv) * dh;
    const int n_v = a.Hkv * dh;
    for (int w = threadIdx.x; w < n_v; w += 256) {
        const int kh = w / dh, d = w % dh;
        pool[a.geom.v_block(a.layer, page, kh) + a.geom.v_elem(slot, d)] = vsrc[w];
    }
}

hipError_t launch_rope_kv(const RopeKvArgs& a, hipStream_t s) {
    if (a.rows <= 0) return hipSuccess;
    if (a.dtype == kF32)
        rope_kv_kernel<float><<<a.rows, 256, 0, s>>>(a);
    else
        rope_kv_kernel<bf16><<<a.rows, 256, 0, s>>>(a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// One workgroup of 1024 threads; thread t owns rows [t * per, (t + 1) * per).
__global__ __launch_bounds__(1024) void compact_rows_kernel(const uint8_t* __restrict__ active, int n_rows,
                                                            int32_t* __restrict__ live, int32_t* __restrict__ row_of,
                                                            int32_t* __restrict__ count_dev,
                                                            uint64_t* __restrict__ mailbox, uint32_t generation) {
    __shared__ int wave_tot[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (n_rows + 1023) / 1024;
    const int r0 = min(n_rows, tid * per), r1 = min(n_rows, r0 + per);
    int mine = 0;
    for (int r = r0; r < r1; ++r) mine += active[r] != 0;
    // exclusive prefix over the 1024 threads: inside a wave by shuffles, across waves through LDS
    int incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int base = 0, total = 0;
    for (int w = 0; w < 16; ++w) {
        if (w < wave) base += wave_tot[w];
        total += wave_tot[w];
    }
    int c = base + incl - mine;
    for (int r = r0; r < r1; ++r) {
        if (active[r] != 0) {
            live[c] = r;
            row_of[r] = c++;
        } else {
            row_of[r] = -1;
        }
    }
    for (int k = total + tid; k < n_rows; k += 1024) live[k] = -1;
    if (tid == 0) {
        *count_dev = total;
        if (mailbox) *(volatile uint64_t*)mailbox = ((uint64_t)generation << 32) | (uint32_t)total;
    }
}

hipError_t launch_compact_rows(const uint8_t* active, int n_rows, int32_t* live, int32_t* row_of,
                               int32_t* count_dev, uint64_t* mailbox, uint32_t generation, hipStream_t s) {
    if (n_rows <= 0) return hipSuccess;
    compact_rows_kernel<<<1, 1024, 0, s>>>(active, n_rows, live, row_of, count_dev, mailbox, generation);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// grid (rollout, layer); copies the K and V blocks of all heads of one page (they are
// contiguous: page_stride elements) in 16-byte pieces.
__global__ __launch_bounds__(256) void fork_copy_kernel(uint4* __restrict__ pool, int64_t page_vec,
                                                        int64_t layer_vec,
                                                        const int32_t* __restrict__ src_page,
                                                        const int32_t* __restrict__ dst_page) {
    const int b = blockIdx.x, layer = blockIdx.y;
    const int sp = src_page[b];
    if (sp < 0) return;
    const uint4* src = pool + layer * layer_vec + (int64_t)sp * page_vec;
    uint4* dst = pool + layer * layer_vec + (int64_t)dst_page[b] * page_vec;
    for (int64_t i = threadIdx.x; i < page_vec; i += 256) dst[i] = src[i];
}

hipError_t launch_fork_copy(void* kv_pool, int dtype, KvGeom geom, int n_layers, const int32_t* src_page,
                            const int32_t* dst_page, int n_rollouts, hipStream_t s) {
    if (n_rollouts <= 0) return hipSuccess;
    const int64_t esz = (int64_t)dtype_size(dtype);
    const int64_t page_vec = geom.page_stride() * esz / 16;  // page_tokens >= 16 keeps this exact
    const int64_t layer_vec = geom.layer_stride() * esz / 16;
    fork_copy_kernel<<<dim3(n_rollouts, n_layers), 256, 0, s>>>((uint4*)kv_pool, page_vec, layer_vec,
                                                               src_page, dst_page);
    return hipGetLastError();
}

}  // namespace rpo
