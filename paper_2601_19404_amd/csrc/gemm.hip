// C[M,N] (op)= A[M,K] * W[N,K]^T with fp32 accumulation: the dense contractions of
// the decoder (QKV, O, gate/up, down, LM head).  Both operands are K-contiguous.
//
//  * gemm_mfma_kernel: bf16 operands on the CDNA4 matrix cores
//    (v_mfma_f32_32x32x16_bf16), LDS-staged 64-deep K slabs, double buffered, the
//    next slab's global loads in flight while the current one is multiplied.
//  * gemm_generic_kernel: any dtype on the vector ALUs (fp32 tiny model, shapes the
//    MFMA kernel does not take).
#include "kernels.hpp"

namespace rpo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------
// generic kernel: 64x64 tile, 16-deep slabs, 256 threads, 4x4 outputs per thread
// ---------------------------------------------------------------------------
template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T* __restrict__ A, int64_t lda,
                                                           const T* __restrict__ W, int64_t ldw,
                                                           void* __restrict__ Cv, int64_t ldc, int M,
                                                           int N, int K) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Ws[BK][BN + 4];
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int tid = threadIdx.x;
    const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += BK) {
        for (int e = tid; e < BM * BK; e += 256) {
            const int r = e / BK, c = e % BK;
            const int gm = m0 + r, gk = k0 + c;
            As[c][r] = (gm < M && gk < K) ? to_f32<T>(A[(int64_t)gm * lda + gk]) : 0.0f;
            const int gn = n0 + r;
            Ws[c][r] = (gn < N && gk < K) ? to_f32<T>(W[(int64_t)gn * ldw + gk]) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < BK; ++c) {
            float av[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[c][tm + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) wv[j] = Ws[c][tn + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + tm + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tn + j;
            if (gn >= N) continue;
            const int64_t o = (int64_t)gm * ldc + gn;
            if (EPI == kEpiStore)
                ((T*)Cv)[o] = from_f32<T>(acc[i][j]);
            else if (EPI == kEpiStoreF32)
                ((float*)Cv)[o] = acc[i][j];
            else
                ((float*)Cv)[o] += acc[i][j];
        }
    }
}

// ---------------------------------------------------------------------------
// MFMA kernel.
//
// Workgroup tile BM x BN, WM x WN waves, each wave owns (BM/WM) x (BN/WN) outputs as
// 32x32 MFMA blocks.  Operand fragments of v_mfma_f32_32x32x16_bf16: lane l holds
// row (l % 32) of its operand and the 8 consecutive K values starting at 8 * (l / 32);
// the 16 accumulator registers of lane l are column (l % 32), rows
// 8 * (i / 4) + 4 * (l / 32) + (i % 4).
// LDS rows are padded by 8 elements (16 bytes) so the 16-byte fragment reads of
// consecutive rows fall into different banks.
// ---------------------------------------------------------------------------
constexpr int kBK = 64;
constexpr int kLdsRow = kBK + 8;

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM* WN * 64) void gemm_mfma_kernel(const bf16* __restrict__ A, int64_t lda,
                                                                const bf16* __restrict__ W, int64_t ldw,
                                                                void* __restrict__ Cv, int64_t ldc,
                                                                int M, int N, int K, int grid_m) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int A_CHUNKS = BM * (kBK / 8) / NT;  // 16-byte pieces per thread and slab
    constexpr int B_CHUNKS = BN * (kBK / 8) / NT;
    static_assert(BM * (kBK / 8) % NT == 0 && BN * (kBK / 8) % NT == 0, "tile/thread mismatch");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* As = (bf16*)smem_raw;                 // [2][BM][kLdsRow]
    bf16* Bs = As + 2 * BM * kLdsRow;           // [2][BN][kLdsRow]

    // Consecutive workgroups walk down M first: the (few) row tiles that share one
    // weight tile run back to back, so the weight tile is fetched from HBM once.
    const int bm = blockIdx.x % grid_m, bn = blockIdx.x / grid_m;
    const int m0 = bm * BM, n0 = bn * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;

    uint4 ra[A_CHUNKS], rb[B_CHUNKS];
    const uint4 zero4 = {0, 0, 0, 0};

    auto load_slab = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int c = tid + i * NT;
            const int r = c >> 3, kc = (c & 7) * 8;
            const int gm = m0 + r, gk = k0 + kc;
            ra[i] = (gm < M && gk < K) ? *(const uint4*)(A + (int64_t)gm * lda + gk) : zero4;
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            const int c = tid + i * NT;
            const int r = c >> 3, kc = (c & 7) * 8;
            const int gn = n0 + r, gk = k0 + kc;
            rb[i] = (gn < N && gk < K) ? *(const uint4*)(W + (int64_t)gn * ldw + gk) : zero4;
        }
    };
    auto store_slab = [&](int buf) {
        bf16* as = As + buf * BM * kLdsRow;
        bf16* bs = Bs + buf * BN * kLdsRow;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int c = tid + i * NT;
            *(uint4*)(as + (c >> 3) * kLdsRow + (c & 7) * 8) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            const int c = tid + i * NT;
            *(uint4*)(bs + (c >> 3) * kLdsRow + (c & 7) * 8) = rb[i];
        }
    };

    f32x16_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    const int nk = (K + kBK - 1) / kBK;
    load_slab(0);
    store_slab(0);
    __syncthreads();
    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_slab((kt + 1) * kBK);
        const bf16* as = As + buf * BM * kLdsRow + (wm * TM + frag_row) * kLdsRow + frag_k;
        const bf16* bs = Bs + buf * BN * kLdsRow + (wn * TN + frag_row) * kLdsRow + frag_k;
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            bf16x8_t af[MI], bfr[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) af[i] = *(const bf16x8_t*)(as + i * 32 * kLdsRow + ks * 16);
#pragma unroll
            for (int j = 0; j < NI; ++j) bfr[j] = *(const bf16x8_t*)(bs + j * 32 * kLdsRow + ks * 16);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_slab(buf ^ 1);
        __syncthreads();
    }

    const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int gn = n0 + wn * TN + j * 32 + col_in;
            if (gn >= N) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int gm = m0 + wm * TM + i * 32 + 8 * (e >> 2) + row_in + (e & 3);
                if (gm >= M) continue;
                const int64_t o = (int64_t)gm * ldc + gn;
                const float v = acc[i][j][e];
                if (EPI == kEpiStore)
                    ((bf16*)Cv)[o] = f32_to_bf16(v);
                else if (EPI == kEpiStoreF32)
                    ((float*)Cv)[o] = v;
                else
                    ((float*)Cv)[o] += v;
            }
        }
    }
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_mfma_cfg(const GemmArgs& a, hipStream_t s) {
    const int gm = ceil_div(a.M, BM), gn = ceil_div(a.N, BN);
    const size_t lds = (size_t)2 * (BM + BN) * kLdsRow * sizeof(bf16);
    const dim3 grid((unsigned)(gm * gn)), block(WM * WN * 64);
#define RPO_GEMM_CASE(E)                                                                              \
    case E: {                                                                                         \
        auto kern = gemm_mfma_kernel<BM, BN, WM, WN, E>;                                              \
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                           (int)lds);                                                 \
        if (e != hipSuccess) return e;                                                                \
        kern<<<grid, block, lds, s>>>((const bf16*)a.A, a.lda, (const bf16*)a.W, a.ldw, a.C, a.ldc,   \
                                      a.M, a.N, a.K, gm);                                             \
        break;                                                                                        \
    }
    switch (a.epilogue) {
        RPO_GEMM_CASE(kEpiStore)
        RPO_GEMM_CASE(kEpiStoreF32)
        RPO_GEMM_CASE(kEpiAddF32)
        default:
            return hipErrorInvalidValue;
    }
#undef RPO_GEMM_CASE
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_generic(const GemmArgs& a, hipStream_t s) {
    const dim3 grid(ceil_div(a.N, 64), ceil_div(a.M, 64));
    switch (a.epilogue) {
        case kEpiStore:
            gemm_generic_kernel<T, kEpiStore><<<grid, 256, 0, s>>>((const T*)a.A, a.lda, (const T*)a.W,
                                                                   a.ldw, a.C, a.ldc, a.M, a.N, a.K);
            break;
        case kEpiStoreF32:
            gemm_generic_kernel<T, kEpiStoreF32><<<grid, 256, 0, s>>>(
                (const T*)a.A, a.lda, (const T*)a.W, a.ldw, a.C, a.ldc, a.M, a.N, a.K);
            break;
        case kEpiAddF32:
            gemm_generic_kernel<T, kEpiAddF32><<<grid, 256, 0, s>>>((const T*)a.A, a.lda, (const T*)a.W,
                                                                    a.ldw, a.C, a.ldc, a.M, a.N, a.K);
            break;
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (a.dtype == kF32) return launch_generic<float>(a, s);
    // 16-byte operand loads: K-contiguous rows whose starts and strides are multiples of 8 elements.
    const bool vec_ok = (a.K % 8 == 0) && (a.lda % 8 == 0) && (a.ldw % 8 == 0) &&
                        ((uintptr_t)a.A % 16 == 0) && ((uintptr_t)a.W % 16 == 0);
    if (a.path == 1 || !vec_ok) return launch_generic<bf16>(a, s);
    if (a.M <= 64) return launch_mfma_cfg<64, 128, 1, 4>(a, s);
    return launch_mfma_cfg<128, 128, 2, 2>(a, s);
}

}  // namespace rpo
