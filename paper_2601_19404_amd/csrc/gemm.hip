// C[M,N] (op)= A[M,K] * W[N,K]^T with fp32 accumulation: the dense contractions of
// the decoder (QKV, O, gate/up, down, LM head).  Both operands are K-contiguous.
//
//  * gemm_dma_kernel / gemm_dma2_kernel: bf16 operands on the CDNA4 matrix cores
//    (v_mfma_f32_32x32x16_bf16).  64-deep K slabs go from global memory straight into LDS
//    (global_load_lds_dwordx4), two to four stages deep; fragments are double-buffered in registers.
//    Tile shapes and what they are for (pick_tile): 256x256 (many-tile problems: prefill / log-prob
//    chunks, wide decode projections), 256x192 / 256x160 (large M with a narrow N, decode gate/up),
//    128x128 and 64x128 (deep-K decode projections, split along K: the fp32 partial sums go to a
//    workspace and a reduction kernel applies the epilogue -- deterministic, no floating-point
//    atomics), 64x64 and 32x128 (shallow-K decode projections, one tile per CU, no K split).
//    (tile, K-split) work items are dealt evenly to the 8 XCDs, neighbouring tiles to the same XCD
//    (each has its own L2).  The wide two-stage tiles run on gemm_dma2_kernel: every MFMA is followed
//    by one fragment read or one load (the matrix pipe never waits behind a burst of memory
//    instructions), the barrier of a slab sits before its last k-step (the next slab's first
//    fragments and the loads of the slab after it go out under that k-step's MFMAs), and when a
//    launch has many rounds of tiles one resident workgroup per CU walks its share of them, the
//    next tile's first loads in flight during the epilogue.
//  * Epilogues ride on the accumulators: residual add, SwiGLU (the kernel reads the weight rows
//    in the order [32 gate | 32 up | 32 gate | ...], so a wave holds matching gate and up
//    columns), rotary embedding + KV page write (QKV projection of a decode step), log-sum-exp
//    and row maxima (LM head).  All but the rotary one and the plain bf16 store multiply with
//    the MFMA operands swapped, which leaves a lane with one row and runs of four columns.
//  * gemm_mfma_kernel: the same tiling with register-staged LDS fills, for K that is not a
//    multiple of 64 (and selectable for comparison).
//  * gemm_generic_kernel: any dtype on the vector ALUs (fp32 tiny model, shapes the
//    MFMA kernels do not take).
#include "kernels.hpp"

namespace rpo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// g * sigmoid(g); the hardware reciprocal (1 ulp) replaces the IEEE division sequence
__device__ inline float silu_f(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

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

// generic SwiGLU projection: act[m, j] = silu(A W_gate^T)[m, j] * (A W_up^T)[m, j]
template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_swiglu_kernel(const T* __restrict__ A, int64_t lda,
                                                                  const T* __restrict__ W, int64_t ldw,
                                                                  T* __restrict__ C, int64_t ldc, int M,
                                                                  int F, int K) {
    const int j = blockIdx.x * 256 + threadIdx.x, m = blockIdx.y;
    if (j >= F) return;
    const T* a = A + (int64_t)m * lda;
    const T* wg = W + (int64_t)j * ldw;
    const T* wu = W + (int64_t)(F + j) * ldw;
    float g = 0.f, u = 0.f;
    for (int k = 0; k < K; ++k) {
        const float av = to_f32<T>(a[k]);
        g = fmaf(av, to_f32<T>(wg[k]), g);
        u = fmaf(av, to_f32<T>(wu[k]), u);
    }
    C[(int64_t)m * ldc + j] = from_f32<T>(g / (1.0f + expf(-g)) * u);
}

// Epilogue shared by the MFMA kernels: lane l holds column (l % 32) and rows
// 8 * (e / 4) + 4 * (l / 32) + (e % 4) of each 32x32 block.
template <int MI, int NI, int TM, int TN, int EPI>
__device__ inline void gemm_epilogue(f32x16_t (&acc)[MI][NI], void* __restrict__ Cv, int64_t ldc, int M, int N,
                                     int m0, int n0, int wm, int wn, int lane, int split) {
    const int col_in = lane & 31, row_in = (lane >> 5) * 4;
    if (EPI == kEpiSwiglu) {
        // blocks (j, j + 1) = (gate, up) of output columns (n0 + wn*TN)/2 + (j/2)*32 + col_in
        bf16* C = (bf16*)Cv;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; j += 2) {
                const int vn = n0 + wn * TN + j * 32;  // virtual column of the gate block
                if (vn + col_in >= N) continue;         // N = 2F is a multiple of 64: pairs are whole
                const int oc = (vn >> 1) + col_in;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int gm = m0 + wm * TM + i * 32 + 8 * (e >> 2) + row_in + (e & 3);
                    if (gm >= M) continue;
                    C[(int64_t)gm * ldc + oc] = f32_to_bf16(silu_f(acc[i][j][e]) * acc[i][j + 1][e]);
                }
            }
        return;
    }
    float* Cp = (float*)Cv + (EPI == kEpiPartial ? (int64_t)split * M * (int64_t)N : 0);
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
                const float v = acc[i][j][e];
                if (EPI == kEpiStore)
                    ((bf16*)Cv)[(int64_t)gm * ldc + gn] = f32_to_bf16(v);
                else if (EPI == kEpiStoreF32)
                    ((float*)Cv)[(int64_t)gm * ldc + gn] = v;
                else if (EPI == kEpiAddF32)
                    ((float*)Cv)[(int64_t)gm * ldc + gn] += v;
                else
                    Cp[(int64_t)gm * N + gn] = v;
            }
        }
    }
}

// Epilogue for accumulators computed with the MFMA operands swapped (the direct-to-LDS kernel): lane l
// holds ROW (l % 32) of each 32x32 block and, per register quad q, the four consecutive columns
// 8 q + 4 (l / 32) .. + 3 -- so the result leaves in 16-byte (fp32) or 8-byte (bf16) pieces.
template <int MI, int NI, int TM, int TN, int EPI, int SW>
__device__ inline void gemm_epilogue_t(f32x16_t (&acc)[MI][NI], void* __restrict__ Cv, int64_t ldc, int M, int N,
                                       int m0, int n0, int wm, int wn, int lane, int split) {
    typedef unsigned short u16x4_t __attribute__((ext_vector_type(4)));
    const int r_in = lane & 31, c_in = (lane >> 5) * 4;
    if (EPI == kEpiSwiglu && SW == 2) {
        // gate and up of output column (block's virtual column)/2 + 8 q + column-in-quad sit in
        // registers 4 q + t and 4 (q + 2) + t of the same block (q = 0, 1)
        bf16* C = (bf16*)Cv;
        const bool vec = (ldc & 3) == 0 && ((uintptr_t)Cv & 7) == 0;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int gm = m0 + wm * TM + i * 32 + r_in;
            if (gm >= M) continue;
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int vn = n0 + wn * TN + j * 32;
                if (vn >= N) continue;  // N = 2F is a multiple of 32: blocks are whole
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    u16x4_t o;
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        o[t] = f32_to_bf16(silu_f(acc[i][j][4 * q + t]) * acc[i][j][4 * (q + 2) + t]).bits;
                    bf16* dst = C + (int64_t)gm * ldc + (vn >> 1) + 8 * q + c_in;
                    if (vec) {
                        *(u16x4_t*)dst = o;
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t) dst[t].bits = o[t];
                    }
                }
            }
        }
        return;
    }
    if (EPI == kEpiSwiglu) {
        // blocks (j, j + 1) = (gate, up) of output columns (n0 + wn*TN + j*32)/2 + column in block
        bf16* C = (bf16*)Cv;
        const bool vec = (ldc & 3) == 0 && ((uintptr_t)Cv & 7) == 0;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int gm = m0 + wm * TM + i * 32 + r_in;
            if (gm >= M) continue;
#pragma unroll
            for (int j = 0; j < NI; j += 2) {
                const int vn = n0 + wn * TN + j * 32;  // virtual column of the gate block
                if (vn >= N) continue;                  // N = 2F is a multiple of 64: pairs are whole
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int oc = (vn >> 1) + 8 * q + c_in;
                    u16x4_t o;
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        o[t] = f32_to_bf16(silu_f(acc[i][j][4 * q + t]) * acc[i][j + 1][4 * q + t]).bits;
                    bf16* dst = C + (int64_t)gm * ldc + oc;
                    if (vec) {
                        *(u16x4_t*)dst = o;
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t) dst[t].bits = o[t];
                    }
                }
            }
        }
        return;
    }
    if (EPI == kEpiStore) {
        bf16* C = (bf16*)Cv;
        const bool vec = (ldc & 3) == 0 && ((uintptr_t)Cv & 7) == 0;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int gm = m0 + wm * TM + i * 32 + r_in;
            if (gm >= M) continue;
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int gn = n0 + wn * TN + j * 32 + 8 * q + c_in;
                    bf16* dst = C + (int64_t)gm * ldc + gn;
                    if (vec && gn + 3 < N) {
                        u16x4_t o;
#pragma unroll
                        for (int t = 0; t < 4; ++t) o[t] = f32_to_bf16(acc[i][j][4 * q + t]).bits;
                        *(u16x4_t*)dst = o;
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (gn + t < N) dst[t] = f32_to_bf16(acc[i][j][4 * q + t]);
                    }
                }
        }
        return;
    }
    // fp32 results: store, accumulate, or K-split partial sums
    const int64_t ld = EPI == kEpiPartial ? (int64_t)N : ldc;
    float* C = (float*)Cv + (EPI == kEpiPartial ? (int64_t)split * M * (int64_t)N : 0);
    const bool vec = (ld & 3) == 0 && ((uintptr_t)C & 15) == 0;
    if (vec && n0 + wn * TN + NI * 32 <= N) {
        // Every column of the wave's blocks exists (the same answer in every lane): straight-line code, no
        // wait between the writes.  Accumulating: all of a row block's reads go out before its first write
        // (the compiler may not move a read of C across a write to C; read and written quad by quad, every
        // quad would wait a full memory round trip: o-projection of an 8192-row chunk 69 -> 51 us).  Reading
        // the next row block ahead of this one's writes as well was measured and gains nothing.
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int gm = m0 + wm * TM + i * 32 + r_in;
            if (gm >= M) continue;
            float* row = C + (int64_t)gm * ld + n0 + wn * TN + c_in;
            float4 c[NI][4];
            if (EPI == kEpiAddF32) {
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) c[j][q] = *(const float4*)(row + j * 32 + 8 * q);
            }
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float4 v = float4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    if (EPI == kEpiAddF32) {
                        v.x += c[j][q].x;
                        v.y += c[j][q].y;
                        v.z += c[j][q].z;
                        v.w += c[j][q].w;
                    }
                    *(float4*)(row + j * 32 + 8 * q) = v;
                }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int gm = m0 + wm * TM + i * 32 + r_in;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int gn = n0 + wn * TN + j * 32 + 8 * q + c_in;
                float* dst = C + (int64_t)gm * ld + gn;
                if (vec && gn + 3 < N) {
                    float4 v = float4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    if (EPI == kEpiAddF32) {
                        const float4 c = *(const float4*)dst;
                        v.x += c.x;
                        v.y += c.y;
                        v.z += c.z;
                        v.w += c.w;
                    }
                    *(float4*)dst = v;
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if (gn + t < N) {
                            if (EPI == kEpiAddF32)
                                dst[t] += acc[i][j][4 * q + t];
                            else
                                dst[t] = acc[i][j][4 * q + t];
                        }
                }
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
constexpr int kXcd = 8;  // XCDs of an MI355X; workgroup i is dispatched to XCD i % 8
// Default direct-to-LDS pipeline shape.  Measured on the prefill gate/up projection: 64-deep slabs
// in two stages beat 32-deep slabs in four stages and four waves of 128x128: not latency-bound.
constexpr int kDmaBK = 64, kDmaStages = 2;

// Column n of the (virtual) output -> row of W.  SwiGLU mode interleaves gate and up rows
// in blocks of 32: virtual columns [64q, 64q+32) are gate rows 32q.., [64q+32, 64q+64) up rows.
// Mode 2 interleaves in blocks of 16 instead (virtual columns [32q, 32q+16) are gate rows 16q..,
// [32q+16, 32q+32) up rows): with the transposed accumulators a lane then holds the gate and the
// up value of an output in one 32x32 block (registers 4 q + t and 4 (q + 2) + t), whatever the
// number of blocks per wave.
template <int SWIGLU>
__device__ inline int weight_row(int n, int F) {
    if (SWIGLU == 0) return n;
    if (SWIGLU == 2) return ((n >> 4) & 1) * F + ((n >> 5) << 4) + (n & 15);
    return ((n >> 5) & 1) * F + ((n >> 6) << 5) + (n & 31);
}

// Tile order shared by the MFMA kernels.  A launch has n_tiles * splits work items (item =
// split * n_tiles + logical tile, n_tiles = grid_m * grid_n: no padding items).  Workgroup ids are
// dealt round-robin to the 8 XCDs, so the ids one XCD sees (i % 8 == x) are mapped to one
// contiguous run of items, the runs as equal as possible: a launch of about one workgroup per
// CU then really puts one on every CU.  Logical tiles walk the grid in column bands of 4 tile
// columns (the last band narrower), each band in blocks of 8 tile rows (the last shorter),
// each block column-major: the ~32 workgroups running together on an XCD share about 8 row slabs
// and 4 weight slabs through its L2.
struct TileCoord {
    int bm, bn, split;
    int ok;  // an int, not a bool: copies of the struct then stay in registers
};
// vb: the virtual block id to map (a workgroup that walks several tiles), or < 0: blockIdx.x.
__device__ inline TileCoord tile_coord(int n_tiles, int splits, int grid_m, int grid_n, int vb = -1) {
    TileCoord t{0, 0, 0, 0};
    const int total = n_tiles * splits;
    const int bid = vb < 0 ? (int)blockIdx.x : vb;
    const int xcd = bid % kXcd;
    const int start = (int)(((int64_t)xcd * total) / kXcd), next = (int)(((int64_t)(xcd + 1) * total) / kXcd);
    const int item = start + bid / kXcd;
    if (item >= next) return t;
    t.split = item / n_tiles;
    int r = item % n_tiles;
    // column band
    const int band_tiles = grid_m * 4, full_bands = grid_n / 4;
    int band = r / band_tiles, width = 4;
    if (band >= full_bands) {
        band = full_bands;
        width = grid_n - full_bands * 4;
    }
    r -= band * band_tiles;
    // block of rows inside the band
    const int full_blocks = grid_m / 8;
    int blk = r / (8 * width), height = 8;
    if (blk >= full_blocks) {
        blk = full_blocks;
        height = grid_m - full_blocks * 8;
    }
    r -= blk * 8 * width;
    t.bm = blk * 8 + r % height;
    t.bn = band * 4 + r / height;
    t.ok = 1;
    return t;
}

// EPI: kEpiStore / kEpiStoreF32 / kEpiAddF32 / kEpiSwiglu write the result; kEpiPartial writes
// fp32 partial sums of its K split to Cv[split][M][N].
template <int BM, int BN, int WM, int WN, int EPI, int SWIGLU>
__global__ __launch_bounds__(WM* WN * 64) void gemm_mfma_kernel(const bf16* __restrict__ A, int64_t lda,
                                                                const bf16* __restrict__ W, int64_t ldw,
                                                                void* __restrict__ Cv, int64_t ldc,
                                                                int M, int N, int K, int grid_m, int grid_n,
                                                                int n_tiles, int splits, int k_per_split, int F) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int A_CHUNKS = BM * (kBK / 8) / NT;  // 16-byte pieces per thread and slab
    constexpr int B_CHUNKS = BN * (kBK / 8) / NT;
    static_assert(BM * (kBK / 8) % NT == 0 && BN * (kBK / 8) % NT == 0, "tile/thread mismatch");
    static_assert(SWIGLU != 1 || NI % 2 == 0, "SwiGLU needs gate/up block pairs inside a wave");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* As = (bf16*)smem_raw;                 // [2][BM][kLdsRow]
    bf16* Bs = As + 2 * BM * kLdsRow;           // [2][BN][kLdsRow]

    const TileCoord tc = tile_coord(n_tiles, splits, grid_m, grid_n);
    if (!tc.ok) return;
    const int m0 = tc.bm * BM, n0 = tc.bn * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int k_begin = tc.split * k_per_split;
    const int k_end = min(K, k_begin + k_per_split);

    // Thread t moves the 16-byte piece (row t / 8 + i * NT / 8, k-chunk t % 8) of each slab.
    // Loads are unconditional (rows beyond M / N are clamped to the last row: their products
    // are never stored; a K tail is zeroed by a select), so the compiler can count the loads in
    // flight and wait only for the older register set.
    constexpr int ROWS_PER_PASS = NT / 8;
    const int ld_row = tid >> 3, ld_k = (tid & 7) * 8;
    // Two register sets: while slab kt is multiplied out of LDS, slab kt+1 sits in one set
    // (about to be written to the other LDS buffer) and slab kt+2 is in flight into the other,
    // so a global load has two slabs of MFMA work to hide behind.
    u32x4_t ra0[A_CHUNKS], rb0[B_CHUNKS], ra1[A_CHUNKS], rb1[B_CHUNKS];
    int64_t a_off[A_CHUNKS], b_off[B_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
        const int gm = min(m0 + ld_row + i * ROWS_PER_PASS, M - 1);
        a_off[i] = (int64_t)gm * lda;
    }
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) {
        const int gn = min(n0 + ld_row + i * ROWS_PER_PASS, N - 1);
        b_off[i] = (int64_t)weight_row<SWIGLU>(gn, F) * ldw;
    }
    const u32x4_t zero4 = {0u, 0u, 0u, 0u};

#define RPO_LOAD_SLAB(RA, RB, k0)                                                                    \
    {                                                                                                \
        const bool k_ok = (k0) + ld_k < k_end;                                                       \
        const int kk = k_ok ? (k0) + ld_k : k_end - 8;                                               \
        _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i) {                                       \
            const u32x4_t v = *(const u32x4_t*)(A + a_off[i] + kk);                                  \
            RA[i] = k_ok ? v : zero4;                                                                \
        }                                                                                            \
        _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i) {                                       \
            const u32x4_t v = *(const u32x4_t*)(W + b_off[i] + kk);                                  \
            RB[i] = k_ok ? v : zero4;                                                                \
        }                                                                                            \
    }
#define RPO_STORE_SLAB(RA, RB, buf)                                                                  \
    {                                                                                                \
        bf16* as_ = As + (buf) * BM * kLdsRow + ld_row * kLdsRow + ld_k;                             \
        bf16* bs_ = Bs + (buf) * BN * kLdsRow + ld_row * kLdsRow + ld_k;                             \
        _Pragma("unroll") for (int i = 0; i < A_CHUNKS; ++i)                                         \
            *(u32x4_t*)(as_ + i * ROWS_PER_PASS * kLdsRow) = RA[i];                                  \
        _Pragma("unroll") for (int i = 0; i < B_CHUNKS; ++i)                                         \
            *(u32x4_t*)(bs_ + i * ROWS_PER_PASS * kLdsRow) = RB[i];                                  \
    }
#define RPO_MULTIPLY_SLAB(buf)                                                                       \
    {                                                                                                \
        const bf16* as = As + (buf) * BM * kLdsRow + (wm * TM + frag_row) * kLdsRow + frag_k;        \
        const bf16* bs = Bs + (buf) * BN * kLdsRow + (wn * TN + frag_row) * kLdsRow + frag_k;        \
        _Pragma("unroll") for (int ks = 0; ks < kBK / 16; ++ks) {                                    \
            bf16x8_t af[MI], bfr[NI];                                                                \
            _Pragma("unroll") for (int i = 0; i < MI; ++i)                                           \
                af[i] = *(const bf16x8_t*)(as + i * 32 * kLdsRow + ks * 16);                         \
            _Pragma("unroll") for (int j = 0; j < NI; ++j)                                           \
                bfr[j] = *(const bf16x8_t*)(bs + j * 32 * kLdsRow + ks * 16);                        \
            _Pragma("unroll") for (int i = 0; i < MI; ++i)                                           \
                _Pragma("unroll") for (int j = 0; j < NI; ++j)                                       \
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0); \
        }                                                                                            \
    }

    f32x16_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    const int nk = (k_end - k_begin + kBK - 1) / kBK;
    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
    // slab s lives in LDS buffer s & 1; odd slabs travel through register set 0, even ones
    // (from slab 2 on) through set 1.  Loads are issued unconditionally (past the last slab
    // they re-read it and the data is dropped) so that every wait for a register set can
    // leave exactly the other set's loads in flight.
#define RPO_SLAB_K(s_) (k_begin + ((s_) < nk ? (s_) : nk - 1) * kBK)
    if (nk > 0) {
        RPO_LOAD_SLAB(ra0, rb0, k_begin);
        RPO_STORE_SLAB(ra0, rb0, 0);
        RPO_LOAD_SLAB(ra0, rb0, RPO_SLAB_K(1));
        RPO_LOAD_SLAB(ra1, rb1, RPO_SLAB_K(2));
        __syncthreads();
        for (int kt = 0; kt < nk; kt += 2) {
            RPO_MULTIPLY_SLAB(0);
            if (kt + 1 < nk) RPO_STORE_SLAB(ra0, rb0, 1);
            RPO_LOAD_SLAB(ra0, rb0, RPO_SLAB_K(kt + 3));
            __syncthreads();
            if (kt + 1 < nk) {
                RPO_MULTIPLY_SLAB(1);
                if (kt + 2 < nk) RPO_STORE_SLAB(ra1, rb1, 0);
            }
            RPO_LOAD_SLAB(ra1, rb1, RPO_SLAB_K(kt + 4));
            __syncthreads();
        }
    }
#undef RPO_SLAB_K

#undef RPO_LOAD_SLAB
#undef RPO_STORE_SLAB
#undef RPO_MULTIPLY_SLAB

    gemm_epilogue<MI, NI, TM, TN, EPI>(acc, Cv, ldc, M, N, m0, n0, wm, wn, lane, tc.split);
}

// ---------------------------------------------------------------------------
// MFMA kernel, direct-to-LDS variant (K a multiple of 64).
//
// Same tiling and epilogues as gemm_mfma_kernel, but the slabs never pass through
// registers: each lane issues global_load_lds_dwordx4, which writes 16 bytes straight
// into LDS at M0 + 16 * lane.  A wave instruction therefore fills 1 KiB = 8 rows of an
// UNPADDED [rows][64] bf16 stage; bank conflicts of the fragment reads are avoided by
// permuting the eight 16-byte pieces of a row: piece p of row r is stored at position
// p ^ g(r), g(r) = (r & 7) ^ ((r >> 3) & 1) (the lane picks its global source piece
// accordingly).  Two LDS stages: the loads of slab kt+1 are issued right after the
// barrier that retires slab kt-1 and land while slab kt is multiplied.  The loads are
// inline assembly (the compiler's own wait-count pass would otherwise wait for every
// outstanding LDS-writing load before each LDS read), so the waits are explicit.
// ---------------------------------------------------------------------------
__device__ inline void dma_load16(const void* gptr, uint32_t lds_byte_addr) {
    asm volatile(
        "s_mov_b32 m0, %1\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, off\n\t"
        :
        : "v"(gptr), "s"(lds_byte_addr)
        : "memory");
}

// Position permutation of the 16-byte pieces of an LDS row (see above), for rows of 8 pieces
// (64-deep slabs) and of 4 pieces (32-deep slabs).  Conflict-free for 16-byte reads of 16
// consecutive rows whether the LDS serves 8 or 16 lanes per cycle.
template <int BK>
__device__ inline int lds_swizzle(int row) {
    if (BK == 64) return (row & 7) ^ ((row >> 3) & 1);
    return ((row >> 2) & 3) ^ (((row >> 1) & 1) << 1);
}

template <int BM, int BN, int WM, int WN, int EPI, int SWIGLU, int BK, int STAGES>
__global__ __launch_bounds__(WM* WN * 64) void gemm_dma_kernel(const bf16* __restrict__ A, int64_t lda,
                                                               const bf16* __restrict__ W, int64_t ldw,
                                                               void* __restrict__ Cv, int64_t ldc, int M,
                                                               int N, int K, int grid_m, int grid_n,
                                                               int n_tiles, int splits, int k_per_split, int F,
                                                               RopeKvArgs rk, LseFuse lf) {
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int PIECES = BK / 8;             // 16-byte pieces per row
    constexpr int ROWS_PER_INST = 64 / PIECES;  // rows one wave instruction fills (1 KiB)
    constexpr int A_INST = BM / ROWS_PER_INST / NW;
    constexpr int B_INST = BN / ROWS_PER_INST / NW;
    constexpr int A_STAGE = BM * BK, B_STAGE = BN * BK;  // elements
    static_assert(BK == 64 || BK == 32, "slab depth");
    static_assert(BM % (ROWS_PER_INST * NW) == 0 && BN % (ROWS_PER_INST * NW) == 0, "tile/wave mismatch");
    static_assert(SWIGLU != 1 || NI % 2 == 0, "SwiGLU needs gate/up block pairs inside a wave");
    static_assert(STAGES >= 2 && STAGES <= 4, "pipeline depth");
    static_assert(EPI != kEpiLse && EPI != kEpiLogitsMax, "these epilogues live on gemm_dma2_kernel");
    // Every epilogue but the rotary one and the plain bf16 store (measured: 2-byte stores of 32
    // neighbouring lanes beat 8-byte stores of 32 rows) multiplies with the operands swapped: the accumulators then
    // hold the transposed block, lane = row of A (l % 32), registers = 16 columns
    // 8 * (e / 4) + 4 * (l / 32) + (e % 4).  Results leave in 16-byte pieces, and reductions along N
    // stay inside a lane (plus one exchange between the lane halves).
    constexpr bool kTrans = EPI != kEpiRope && EPI != kEpiStore;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* As = (bf16*)smem_raw;             // [STAGES][BM][BK]
    bf16* Bs = As + STAGES * A_STAGE;       // [STAGES][BN][BK]
    const uint32_t lds_a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem_raw;
    const uint32_t lds_b = lds_a + STAGES * A_STAGE * 2;

    const TileCoord tc = tile_coord(n_tiles, splits, grid_m, grid_n);
    if (!tc.ok) return;
    const int m0 = tc.bm * BM, n0 = tc.bn * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int k_begin = tc.split * k_per_split;
    const int k_end = min(K, k_begin + k_per_split);
    const int nk = (k_end - k_begin) / BK;

    // Load addressing.  Instruction j of this wave fills row group rg = j * NW + wave; this lane's
    // row is rg * ROWS_PER_INST + lane / PIECES and it stores at position lane % PIECES, i.e. it
    // fetches piece (lane % PIECES) ^ swizzle(row).
    const bf16* a_src[A_INST];
    const bf16* b_src[B_INST];
#pragma unroll
    for (int j = 0; j < A_INST; ++j) {
        const int row = (j * NW + wave) * ROWS_PER_INST + lane / PIECES;
        const int piece = (lane % PIECES) ^ lds_swizzle<BK>(row);
        a_src[j] = A + (int64_t)min(m0 + row, M - 1) * lda + piece * 8 + k_begin;
    }
#pragma unroll
    for (int j = 0; j < B_INST; ++j) {
        const int row = (j * NW + wave) * ROWS_PER_INST + lane / PIECES;
        const int piece = (lane % PIECES) ^ lds_swizzle<BK>(row);
        b_src[j] = W + (int64_t)weight_row<SWIGLU>(min(n0 + row, N - 1), F) * ldw + piece * 8 + k_begin;
    }
    // Narrow tiles: many workgroups share each operand slab (all row tiles of a column tile read the
    // same weight rows, all column tiles of a row tile the same activations).  Each workgroup walks
    // K from its own starting slab, so that the workgroups running together ask the L2 for
    // different lines instead of the same ones at the same time.
    const int k_rot = (BM <= 64 && nk > 0) ? (tc.bm * 5 + tc.bn * 3) % nk : 0;
    // slab s_ (clamped to the last one: loads past the end are redundant, never read) -> stage
#define RPO_DMA_SLAB(s_)                                                                                 \
    {                                                                                                    \
        int sl_ = ((s_) < nk ? (s_) : nk - 1) + k_rot;                                                   \
        sl_ = sl_ >= nk ? sl_ - nk : sl_;                                                                \
        const int st_ = (s_) % STAGES;                                                                   \
        _Pragma("unroll") for (int j = 0; j < A_INST; ++j)                                               \
            dma_load16(a_src[j] + sl_ * BK, lds_a + (st_ * A_STAGE + (j * NW + wave) * 512) * 2);        \
        _Pragma("unroll") for (int j = 0; j < B_INST; ++j)                                               \
            dma_load16(b_src[j] + sl_ * BK, lds_b + (st_ * B_STAGE + (j * NW + wave) * 512) * 2);        \
    }

    f32x16_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Fragment addressing: row = 32-aligned base + lane % 32, so the swizzle depends on the lane only.
    const int frag_row = lane & 31;
    const int frag_g = lds_swizzle<BK>(frag_row);
    const int frag_half = lane >> 5;
    // STAGES - 1 slabs are in flight ahead of the one being multiplied; after issuing slab
    // kt + STAGES - 1 a wave waits until all but the newest STAGES - 2 slabs' loads have landed.
    constexpr int kInFlight = (STAGES - 2) * (A_INST + B_INST);
    if (nk > 0) {
#pragma unroll
        for (int s0 = 0; s0 < STAGES - 1; ++s0) RPO_DMA_SLAB(s0);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kInFlight) : "memory");
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int stage = kt % STAGES;
            RPO_DMA_SLAB(kt + STAGES - 1);  // into the stage whose slab (kt - 1) everyone has finished reading
            const bf16* as = As + stage * A_STAGE + (wm * TM + frag_row) * BK;
            const bf16* bs = Bs + stage * B_STAGE + (wn * TN + frag_row) * BK;
            // Fragments are double-buffered in registers: the LDS reads of k-step ks + 1 are issued
            // before the MFMAs of k-step ks, so the LDS pipe and the matrix pipe work at the same time.
            constexpr int KS = BK / 16;
            bf16x8_t af[2][MI], bfr[2][NI];
            {
                const int piece = (frag_half ^ frag_g) * 8;
#pragma unroll
                for (int i = 0; i < MI; ++i) af[0][i] = *(const bf16x8_t*)(as + i * 32 * BK + piece);
#pragma unroll
                for (int j = 0; j < NI; ++j) bfr[0][j] = *(const bf16x8_t*)(bs + j * 32 * BK + piece);
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int cur = ks & 1, nxt = cur ^ 1;
                if (ks + 1 < KS) {
                    const int piece = (((ks + 1) * 2 + frag_half) ^ frag_g) * 8;
#pragma unroll
                    for (int i = 0; i < MI; ++i) af[nxt][i] = *(const bf16x8_t*)(as + i * 32 * BK + piece);
#pragma unroll
                    for (int j = 0; j < NI; ++j) bfr[nxt][j] = *(const bf16x8_t*)(bs + j * 32 * BK + piece);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = kTrans ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][j], af[cur][i], acc[i][j], 0, 0, 0)
                                           : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][i], bfr[cur][j], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kInFlight) : "memory");
            __syncthreads();
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // drain the redundant tail loads before LDS is released
    }
#undef RPO_DMA_SLAB
    if constexpr (EPI == kEpiRope) {
        // The tile is BM rows of one head (BN = head_dim = 128, checked by the launcher).  The
        // accumulators go to LDS as fp32 [BM][BN + 1]; the rotation pairs (i, i + 64) of a row
        // then sit in one place whatever wave produced them.  q is rotated and stored to C, k is
        // rotated and stored to its page slot, v is stored transposed into its page.
        static_assert(EPI != kEpiRope || (BN == 128 && WM == 1 && (BM == 32 || BM == 64) && NW == 4), "one head per tile");
        constexpr int LD = BN + 1;
        float* tile = (float*)smem_raw;
        int* row_pos = (int*)(tile + BM * LD);   // position, or -1: row beyond M / not active
        int64_t* row_page = (int64_t*)(row_pos + BM + (BM & 1));
        __syncthreads();  // every wave's tail loads have landed; the stages can be overwritten
        {
            const int col = wn * TN + (lane & 31), row_in = (lane >> 5) * 4;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    tile[(i * 32 + 8 * (e >> 2) + row_in + (e & 3)) * LD + col] = acc[i][0][e];
        }
        if (tid < BM) {
            const int r = m0 + tid;
            int pos = -1;
            int64_t page = 0;
            const int seq = r < M ? (rk.row_seq ? rk.row_seq[r] : r) : -1;
            if (seq >= 0 && !(rk.active && !rk.active[r])) {
                const SeqDesc sd = rk.seqs[seq];
                pos = sd.pos0 + (rk.single_row ? 0 : r - sd.row_start) + rk.pos_add;
                page = rk.tables[sd.table_off + pos / rk.geom.page_tokens];
            }
            row_pos[tid] = pos;
            row_page[tid] = page;
        }
        __syncthreads();
        const int head = n0 / BN;
        const int pt = rk.geom.page_tokens;
        bf16* pool = (bf16*)rk.kv_pool;
        if (head < rk.Hq + rk.Hkv) {
            const int i = tid & 63;
#pragma unroll
            for (int it = 0; it < BM / 4; ++it) {
                const int row = it * 4 + (tid >> 6);
                const int gm = m0 + row;
                if (gm >= M) continue;
                const int pos = row_pos[row];
                const float x1 = tile[row * LD + i], x2 = tile[row * LD + i + 64];
                bf16* dst;
                float y1 = x1, y2 = x2;
                if (pos >= 0) {
                    const float2 cs = *(const float2*)(rk.rope + ((int64_t)pos * 64 + i) * 2);
                    y1 = x1 * cs.x - x2 * cs.y;
                    y2 = x2 * cs.x + x1 * cs.y;
                }
                if (head < rk.Hq) {
                    dst = (bf16*)Cv + (int64_t)gm * ldc + n0;  // a finished rollout keeps an unrotated q
                } else {
                    if (pos < 0) continue;
                    dst = pool + rk.geom.k_block(rk.layer, row_page[row], head - rk.Hq) + (int64_t)(pos % pt) * BN;
                }
                dst[i] = f32_to_bf16(y1);
                dst[i + 64] = f32_to_bf16(y2);
            }
        } else {
            // a wave writes 64 consecutive channels of one row: 2-byte pieces 16 bytes apart (8 lines)
            const int d = tid & (BN - 1);
#pragma unroll
            for (int it = 0; it < BM / 2; ++it) {
                const int row = it * 2 + (tid >> 7);
                const int pos = row_pos[row];
                if (pos < 0) continue;
                pool[rk.geom.v_block(rk.layer, row_page[row], head - rk.Hq - rk.Hkv) + rk.geom.v_elem(pos % pt, d)] =
                    f32_to_bf16(tile[row * LD + d]);
            }
        }
    } else {
        if constexpr (kTrans)
            gemm_epilogue_t<MI, NI, TM, TN, EPI, SWIGLU>(acc, Cv, ldc, M, N, m0, n0, wm, wn, lane, tc.split);
        else
            gemm_epilogue<MI, NI, TM, TN, EPI>(acc, Cv, ldc, M, N, m0, n0, wm, wn, lane, tc.split);
    }
}

// ---------------------------------------------------------------------------
// Direct-to-LDS kernel of the wide tiles, S stages (2, or 3 where the tile leaves room in the 160 KiB
// of LDS).  A workgroup walks over several tiles (virtual block ids blockIdx.x, blockIdx.x + gridDim.x,
// ...): the loads of the next tile's first S slabs go out during the last S slabs of the current one
// (none after the workgroup's last tile), and inside a slab every MFMA is followed by one fragment read
// / one load so that the matrix pipe never waits behind a burst of memory instructions.
// ---------------------------------------------------------------------------
__device__ inline void dma_load16_s(const void* sbase, uint32_t voff, uint32_t lds_byte_addr) {
    asm volatile(
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, %1\n\t"
        :
        : "v"(voff), "s"(sbase), "s"(lds_byte_addr)
        : "memory");
}

template <int MI, int NI, int TM, int TN, int BN, int WN, int EPI, int SWIGLU>
__device__ inline void dma2_epilogue(f32x16_t (&acc)[MI][NI], void* __restrict__ Cv, int64_t ldc, int M, int N, int m0,
                                     int n0, int wm, int wn, int lane, int split, const LseFuse& lf) {
    constexpr bool kTrans = EPI != kEpiStore;
    if constexpr (EPI == kEpiLse) {
        const int half = lane >> 5;
        const int blk = (n0 / BN) * WN + wn;
        const int cbase = n0 + wn * TN;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int r = m0 + wm * TM + i * 32 + (lane & 31);
            const int tgt = r < M ? lf.target[r] : -1;
            float mx = -INFINITY, zt = 0.f;
            bool have = false;
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int col = cbase + j * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
                    const float v = col < N ? acc[i][j][e] : -INFINITY;
                    acc[i][j][e] = v;
                    mx = fmaxf(mx, v);
                    if (col == tgt) {
                        zt = v;
                        have = true;
                    }
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float muse = mx == -INFINITY ? 0.f : mx;
            const float nb = -muse * lf.k2;
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i][j][e], lf.k2, nb));
            sum += __shfl_xor(sum, 32, 64);
            if (r < M) {
                if (half == 0) {
                    float* p = lf.part + ((int64_t)r * lf.blocks + blk) * 2;
                    p[0] = mx;
                    p[1] = sum;
                }
                if (have) lf.target_logit[r] = zt;
            }
        }
    } else if constexpr (EPI == kEpiLogitsMax) {
        // transposed accumulators: a lane owns a row and, per register quad, four consecutive columns
        const int half = lane >> 5;
        const int blk = (n0 / BN) * WN + wn;
        const int cbase = n0 + wn * TN;
        float* C = (float*)Cv;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int r = m0 + wm * TM + i * 32 + (lane & 31);
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = cbase + j * 32 + 8 * q + 4 * half;
                    if (r < M && col < N) {  // N is a multiple of 4 (checked by the launcher): whole quads
                        const float4 v = float4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                                                acc[i][j][4 * q + 3]};
                        *(float4*)(C + (int64_t)r * ldc + col) = v;
                        mx = fmaxf(fmaxf(mx, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
                    }
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            if (r < M && half == 0) lf.part[(int64_t)r * lf.blocks + blk] = mx;
        }
    } else {
        if constexpr (kTrans)
            gemm_epilogue_t<MI, NI, TM, TN, EPI, SWIGLU>(acc, Cv, ldc, M, N, m0, n0, wm, wn, lane, split);
        else
            gemm_epilogue<MI, NI, TM, TN, EPI>(acc, Cv, ldc, M, N, m0, n0, wm, wn, lane, split);
    }
}

template <int BM, int BN, int WM, int WN, int EPI, int SWIGLU, int S = 2>
__global__ __launch_bounds__(WM* WN * 64) void gemm_dma2_kernel(const bf16* __restrict__ A, int64_t lda,
                                                                const bf16* __restrict__ W, int64_t ldw,
                                                                void* __restrict__ Cv, int64_t ldc, int M,
                                                                int N, int K, int grid_m, int grid_n,
                                                                int n_tiles, int splits, int k_per_split, int F,
                                                                int n_vblocks, LseFuse lf) {
    constexpr int BK = 64, KS = 4;
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int A_INST = BM / 8 / NW, B_INST = BN / 8 / NW;  // a wave instruction fills 8 rows (1 KiB)
    constexpr int A_STAGE = BM * BK, B_STAGE = BN * BK;        // elements
    constexpr int N_INST = A_INST + B_INST;
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile/wave mismatch");
    static_assert(EPI != kEpiRope, "no LDS-staged epilogue here");
    constexpr bool kTrans = EPI != kEpiStore;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* As = (bf16*)smem_raw;        // [S][BM][BK]
    bf16* Bs = As + S * A_STAGE;       // [S][BN][BK]
    const uint32_t lds_a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem_raw;
    const uint32_t lds_b = lds_a + S * A_STAGE * 2;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    int vb = blockIdx.x;
    TileCoord tc = tile_coord(n_tiles, splits, grid_m, grid_n, vb);
    if (!tc.ok) return;

    // Load addressing: instruction j of this wave fills rows (j * NW + wave) * 8 + lane / 8 of a stage;
    // the lane stores at position lane % 8 and therefore fetches piece (lane % 8) ^ swizzle(row).  The
    // address is a per-tile uniform base (scalar registers) plus a 32-bit per-lane byte offset.
    struct Src {
        const bf16* a_base;
        const bf16* b_base;
        uint32_t a_off[A_INST], b_off[B_INST];
        int nk;
    };
    auto setup = [&](const TileCoord& t, Src& o) {
        const int m0 = t.bm * BM, n0 = t.bn * BN;
        const int k_begin = t.split * k_per_split;
        const int k_end = min(K, k_begin + k_per_split);
        o.nk = (k_end - k_begin) / BK;
        o.a_base = A + (int64_t)m0 * lda + k_begin;
        o.b_base = W + k_begin;
#pragma unroll
        for (int j = 0; j < A_INST; ++j) {
            const int row = (j * NW + wave) * 8 + (lane >> 3);
            const int piece = (lane & 7) ^ lds_swizzle<BK>(row);
            o.a_off[j] = (uint32_t)(((int64_t)min(row, M - 1 - m0) * lda + piece * 8) * 2);
        }
#pragma unroll
        for (int j = 0; j < B_INST; ++j) {
            const int row = (j * NW + wave) * 8 + (lane >> 3);
            const int piece = (lane & 7) ^ lds_swizzle<BK>(row);
            o.b_off[j] = (uint32_t)(((int64_t)weight_row<SWIGLU>(min(n0 + row, N - 1), F) * ldw + piece * 8) * 2);
        }
    };
    // instruction t (A first, then B) of slab sl of tile source o into stage st
    auto dma_one = [&](const Src& o, int sl, int st, int t, int on) __attribute__((always_inline)) {
        if (!on) return;  // uniform
        if (t < A_INST)
            dma_load16_s(o.a_base + sl * BK, o.a_off[t], lds_a + (st * A_STAGE + (t * NW + wave) * 512) * 2);
        else
            dma_load16_s(o.b_base + sl * BK, o.b_off[t - A_INST], lds_b + (st * B_STAGE + ((t - A_INST) * NW + wave) * 512) * 2);
    };

    Src cur;
    setup(tc, cur);
    f32x16_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    const int frag_row = lane & 31;
    const int frag_g = lds_swizzle<BK>(frag_row);
    const int frag_half = lane >> 5;
    const int a_frag = (wm * TM + frag_row) * BK, b_frag = (wn * TN + frag_row) * BK;
    const int piece0 = (frag_half ^ frag_g) * 8;
    bf16x8_t af[2][MI], bfr[2][NI];

#pragma unroll
    for (int sl = 0; sl < S; ++sl)
#pragma unroll
        for (int t = 0; t < N_INST; ++t) dma_one(cur, sl, sl, t, 1);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 1) * N_INST) : "memory");
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NI; ++j) bfr[0][j] = *(const bf16x8_t*)(Bs + b_frag + j * 32 * BK + piece0);
#pragma unroll
    for (int i = 0; i < MI; ++i) af[0][i] = *(const bf16x8_t*)(As + a_frag + i * 32 * BK + piece0);

    // One slab (g = running slab count of this workgroup: stage g & 1).  The loads that go out in its
    // last k-step fetch slab dma_sl of the tile `cur` describes, into this slab's stage.
    auto slab_body = [&](const int stage, const int dma_sl, const int on) __attribute__((always_inline)) {
        const int stage1 = stage + 1 == S ? 0 : stage + 1;
        const bf16* as = As + stage * A_STAGE + a_frag;
        const bf16* bs = Bs + stage * B_STAGE + b_frag;
#pragma unroll
        for (int ks = 0; ks < KS - 1; ++ks) {
            const int c = ks & 1, n = c ^ 1;
            const int piece = (((ks + 1) * 2 + frag_half) ^ frag_g) * 8;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const int t = i * NI + j;
                    acc[i][j] = kTrans ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[c][j], af[c][i], acc[i][j], 0, 0, 0)
                                       : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[c][i], bfr[c][j], acc[i][j], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (t < NI) bfr[n][t] = *(const bf16x8_t*)(bs + t * 32 * BK + piece);
                    else if (t < NI + MI) af[n][t - NI] = *(const bf16x8_t*)(as + (t - NI) * 32 * BK + piece);
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
        // Last k-step: its fragments are in registers.  Once every wave's are, this stage is free, and the
        // following slab has landed in the other stage.
        constexpr int c = (KS - 1) & 1, n = c ^ 1;
        // the S - 2 slabs after the next one may still be in flight -- unless the loads have stopped (tail of the
        // workgroup's last tile): then everything outstanding is waited for
        if (S > 2 && on)
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((S - 2) * N_INST) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __syncthreads();
        const bf16* as1 = As + stage1 * A_STAGE + a_frag;
        const bf16* bs1 = Bs + stage1 * B_STAGE + b_frag;
        constexpr int kPer = (N_INST + MI * NI - 1) / (MI * NI);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int t = i * NI + j;
                acc[i][j] = kTrans ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[c][j], af[c][i], acc[i][j], 0, 0, 0)
                                   : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[c][i], bfr[c][j], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (t < NI) bfr[n][t] = *(const bf16x8_t*)(bs1 + t * 32 * BK + piece0);
                else if (t < NI + MI) af[n][t - NI] = *(const bf16x8_t*)(as1 + (t - NI) * 32 * BK + piece0);
#pragma unroll
                for (int d = 0; d < kPer; ++d)
                    if (t * kPer + d < N_INST) dma_one(cur, dma_sl, stage, t * kPer + d, on);
                __builtin_amdgcn_sched_barrier(0);
            }
    };

    // this workgroup's tiles: virtual blocks blockIdx.x + i * gridDim.x while they map to a work item
    int n_my = 0;
    {
        const int total = n_tiles * splits;
        const int xcd = blockIdx.x % kXcd;
        const int cnt = (int)(((int64_t)(xcd + 1) * total) / kXcd) - (int)(((int64_t)xcd * total) / kXcd);
        const int slot = blockIdx.x / kXcd, wpx = gridDim.x / kXcd;
        if (slot < cnt) n_my = (cnt - slot + wpx - 1) / wpx;
    }
    int stage = 0;
#pragma clang loop unroll(disable)
    for (int it = 0; it < n_my; ++it) {
        // the tile after this one (after the last one no loads go out)
        const bool last = it + 1 == n_my;
        TileCoord ntc = tc;
        if (!last) ntc = tile_coord(n_tiles, splits, grid_m, grid_n, vb + (int)gridDim.x);
        const int nk = cur.nk;  // >= S (checked by the launcher)
#pragma clang loop unroll(disable)
        for (int kt = 0; kt < nk; ++kt) {
            if (kt == nk - S && !last) setup(ntc, cur);  // this tile's loads are all out: the addresses become the next tile's
            slab_body(stage, kt + S < nk ? kt + S : kt + S - nk, (kt + S < nk || !last) ? 1 : 0);
            stage = stage + 1 == S ? 0 : stage + 1;
        }
        dma2_epilogue<MI, NI, TM, TN, BN, WN, EPI, SWIGLU>(acc, Cv, ldc, M, N, tc.bm * BM, tc.bn * BN, wm, wn, lane, tc.split, lf);
        tc = ntc;
        vb += (int)gridDim.x;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Sum the K-split partials [splits][M][N] and apply the epilogue.  One thread per output
// element (per gate/up pair in SwiGLU mode); partial sums are added in split order.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(const float* __restrict__ P, int splits,
                                                                 int M, int N, void* __restrict__ Cv,
                                                                 int64_t ldc) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t plane = (int64_t)M * N;
    if (EPI == kEpiSwiglu) {
        const int F = N / 2;
        if (idx >= (int64_t)M * F) return;
        const int m = (int)(idx / F), oc = (int)(idx % F);
        const int vg = ((oc >> 5) << 6) + (oc & 31);  // virtual gate column; up is 32 further
        float g = 0.f, u = 0.f;
        for (int z = 0; z < splits; ++z) {
            g += P[z * plane + (int64_t)m * N + vg];
            u += P[z * plane + (int64_t)m * N + vg + 32];
        }
        ((bf16*)Cv)[(int64_t)m * ldc + oc] = f32_to_bf16(silu_f(g) * u);
        return;
    }
    if (idx >= plane) return;
    const int m = (int)(idx / N), n = (int)(idx % N);
    float v = 0.f;
    for (int z = 0; z < splits; ++z) v += P[z * plane + idx];
    const int64_t o = (int64_t)m * ldc + n;
    if (EPI == kEpiStore)
        ((bf16*)Cv)[o] = f32_to_bf16(v);
    else if (EPI == kEpiStoreF32)
        ((float*)Cv)[o] = v;
    else
        ((float*)Cv)[o] += v;
}

// K-split reduction fused with the residual add and the following RMSNorm: one workgroup per
// row; x[m, :] += sum_z P[z][m, :], then h[m, :] = x / sqrt(mean(x^2) + eps) * gain.
__global__ __launch_bounds__(256) void gemm_splitk_reduce_norm_kernel(const float* __restrict__ P, int splits,
                                                                      int M, int N, float* __restrict__ X,
                                                                      int64_t ldc, const bf16* __restrict__ gain,
                                                                      float eps, bf16* __restrict__ H) {
    // N is a multiple of 4 (checked by the launcher): each thread owns float4 column groups
    // tid, tid + 256, ... of the row, at most 8 of them (N <= 8192).
    constexpr int kMaxVec = 8;
    __shared__ float part[4];
    const int m = blockIdx.x, tid = threadIdx.x;
    const int64_t plane = (int64_t)M * N;
    const int nvec = N >> 2;
    float4 v[kMaxVec];
    float ss = 0.f;
    float4* xrow = (float4*)(X + (int64_t)m * ldc);
    const float4* prow = (const float4*)(P + (int64_t)m * N);
#pragma unroll
    for (int i = 0; i < kMaxVec; ++i) {
        const int c = tid + i * 256;
        if (c < nvec) {
            float4 acc = xrow[c];
            // eight partial sums are requested at a time, then added in split order
            for (int z0 = 0; z0 < splits; z0 += 8) {
                float4 p[8];
#pragma unroll
                for (int z = 0; z < 8; ++z)
                    if (z0 + z < splits) p[z] = prow[((z0 + z) * plane >> 2) + c];
#pragma unroll
                for (int z = 0; z < 8; ++z)
                    if (z0 + z < splits) {
                        acc.x += p[z].x;
                        acc.y += p[z].y;
                        acc.z += p[z].z;
                        acc.w += p[z].w;
                    }
            }
            xrow[c] = acc;
            v[i] = acc;
            ss += (acc.x * acc.x + acc.y * acc.y) + (acc.z * acc.z + acc.w * acc.w);
        }
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) part[tid >> 6] = ss;
    __syncthreads();
    const float tot = (part[0] + part[1]) + (part[2] + part[3]);
    const float inv = 1.0f / sqrtf(tot / (float)N + eps);
    typedef unsigned short u16x4_t __attribute__((ext_vector_type(4)));
    const u16x4_t* grow = (const u16x4_t*)gain;
    u16x4_t* hrow = (u16x4_t*)(H + (int64_t)m * N);
#pragma unroll
    for (int i = 0; i < kMaxVec; ++i) {
        const int c = tid + i * 256;
        if (c < nvec) {
            const u16x4_t g = grow[c];
            u16x4_t o;
            o.x = f32_to_bf16(v[i].x * inv * bf16_to_f32(bf16{g.x})).bits;
            o.y = f32_to_bf16(v[i].y * inv * bf16_to_f32(bf16{g.y})).bits;
            o.z = f32_to_bf16(v[i].z * inv * bf16_to_f32(bf16{g.z})).bits;
            o.w = f32_to_bf16(v[i].w * inv * bf16_to_f32(bf16{g.w})).bits;
            hrow[c] = o;
        }
    }
}

// K-split reduction of the QKV projection fused with the rotary embedding and the KV page
// write: one workgroup per token row sums the partials into LDS (fp32), rotates q and k pairs
// (i, i + dh/2) by the row's position, stores q back to the activation buffer and k, v into
// the row's page slot (v transposed).
__global__ __launch_bounds__(256) void gemm_splitk_reduce_rope_kernel(const float* __restrict__ P, int splits,
                                                                      int M, int N, RopeKvArgs a) {
    extern __shared__ float rowsum[];  // [N]
    const int r = blockIdx.x, tid = threadIdx.x;
    const int64_t plane = (int64_t)M * N;
    for (int c = tid; c < N; c += 256) {
        float acc = 0.f;
        for (int z = 0; z < splits; ++z) acc += P[z * plane + (int64_t)r * N + c];
        rowsum[c] = acc;
    }
    __syncthreads();
    bf16* row = (bf16*)a.qkv + (int64_t)r * N;
    const int dh = a.dh, half = dh / 2;
    const int seq = a.row_seq ? a.row_seq[r] : r;
    if (seq < 0 || (a.active && !a.active[r])) {  // finished rollout / padding row: keep q defined, append nothing
        for (int c = tid; c < a.Hq * dh; c += 256) row[c] = f32_to_bf16(rowsum[c]);
        return;
    }
    const SeqDesc sd = a.seqs[seq];
    const int pos = sd.pos0 + (a.single_row ? 0 : r - sd.row_start) + a.pos_add;
    const int pt = a.geom.page_tokens;
    const int64_t page = a.tables[sd.table_off + pos / pt];
    const int slot = pos % pt;
    bf16* pool = (bf16*)a.kv_pool;
    const float* cs = a.rope + (int64_t)pos * half * 2;
    const int n_rot = (a.Hq + a.Hkv) * half;
    for (int w = tid; w < n_rot; w += 256) {
        const int head = w / half, i = w % half;
        const float c = cs[2 * i], s = cs[2 * i + 1];
        const float x1 = rowsum[head * dh + i], x2 = rowsum[head * dh + i + half];
        const bf16 y1 = f32_to_bf16(x1 * c - x2 * s), y2 = f32_to_bf16(x2 * c + x1 * s);
        if (head < a.Hq) {
            row[head * dh + i] = y1;
            row[head * dh + i + half] = y2;
        } else {
            bf16* kdst = pool + a.geom.k_block(a.layer, page, head - a.Hq) + (int64_t)slot * dh;
            kdst[i] = y1;
            kdst[i + half] = y2;
        }
    }
    const int v0 = (a.Hq + a.Hkv) * dh;
    for (int w = tid; w < a.Hkv * dh; w += 256) {
        const int kh = w / dh, d = w % dh;
        pool[a.geom.v_block(a.layer, page, kh) + a.geom.v_elem(slot, d)] = f32_to_bf16(rowsum[v0 + w]);
    }
}

// ---------------------------------------------------------------------------
// launch logic
// ---------------------------------------------------------------------------
namespace {

struct TileCfg {
    int id;  // KernelId base (store variant)
    int bm, bn;
};

bool mfma_ok(const GemmArgs& a) {
    // 16-byte operand loads: K-contiguous rows whose starts and strides are multiples of 8 elements.
    const bool vec_ok = (a.K % 8 == 0) && (a.lda % 8 == 0) && (a.ldw % 8 == 0) &&
                        ((uintptr_t)a.A % 16 == 0) && ((uintptr_t)a.W % 16 == 0);
    if (a.dtype != kBF16 || a.path == 1 || !vec_ok) return false;
    if (a.epilogue == kEpiSwiglu && (a.N % 64 != 0)) return false;  // N = 2F, F a multiple of 32
    return true;
}

// The rotary epilogue of the narrow kernel: one head per 128-column tile, rows stored with stride N.
bool rope_direct(const GemmArgs& a) {
    return a.rope && a.epilogue == kEpiStore && a.rope->dh == 128 && a.ldc == a.N && a.K % kBK == 0 &&
           a.N == (a.rope->Hq + 2 * a.rope->Hkv) * 128 && a.path != 2;
}

TileCfg pick_tile(const GemmArgs& a) {
    if (a.path >= 16) {  // tuning aid: a fixed tile shape
        switch (a.path - 16) {
            case kKidGemm256: return TileCfg{kKidGemm256, 256, 256};
            case kKidGemm128: return TileCfg{kKidGemm128, 128, 128};
            case kKidGemm32: return TileCfg{kKidGemm32, 32, 128};
            case kKidGemm64x64: return TileCfg{kKidGemm64x64, 64, 64};
            case kKidGemm256x160:  // fused gate/up only
                if (a.epilogue == kEpiSwiglu && a.K % kBK == 0 && (a.N / 2) % 16 == 0)
                    return TileCfg{kKidGemm256x160, 256, 160};
                return TileCfg{kKidGemm256, 256, 256};
            case kKidGemm256x192:  // its fused gate/up epilogue exists on the direct-to-LDS kernel only
                if (a.epilogue != kEpiSwiglu || (a.K % kBK == 0 && (a.N / 2) % 16 == 0))
                    return TileCfg{kKidGemm256x192, 256, 192};
                return TileCfg{kKidGemm256, 256, 256};
            default: return TileCfg{kKidGemm64, 64, 128};
        }
    }
    // Measured on MI355X: the 8-wave 256x256 tile wins whenever it yields at least ~half a
    // chip of workgroups.  Smaller problems are bound by what one CU can load per unit time
    // (every CU has to pull operands): with a shallow K, narrow tiles without K splitting and a
    // four-deep load pipeline beat wider tiles whose K-split partial sums need a second kernel;
    // with a deep K, 128x128 tiles split along K.
    const int t256 = ceil_div(a.M, 256) * ceil_div(a.N, 256);
    // The gate/up projection of a decode step: one round of fewer 256x256 tiles than CUs; 256x192
    // tiles still fit one round and each is a quarter cheaper.
    if (a.epilogue == kEpiSwiglu && a.M > 128 && t256 >= 128 && t256 <= 256 && a.K % kBK == 0 && a.path != 2 &&
        (a.N / 2) % 16 == 0 && ceil_div(a.M, 256) * ceil_div(a.N, 192) <= 256) {
        // 256x160 tiles (four waves of 64x160, three stages) still fit one round and put work on more CUs.
        // Measured with weights streamed from HBM: K = 1536, N = 17920, 512 rows: 39.2 -> 34.3 us;
        // K = 3584, N = 37888, 256 rows: 87.5 -> 78.8 us.
        if (a.K >= 3 * kBK && ceil_div(a.M, 256) * ceil_div(a.N, 160) <= 256) return TileCfg{kKidGemm256x160, 256, 160};
        return TileCfg{kKidGemm256x192, 256, 192};
    }
    // up to 128 rows a 256-row tile multiplies mostly padding
    if (a.epilogue == kEpiSwiglu && a.M > 64 && a.M <= 128 && t256 >= 128) return TileCfg{kKidGemm128, 128, 128};
    if (a.M > 512 || (a.M > 64 && t256 >= 128)) {
        // Workgroups run in rounds of one per CU.  A 256x192 tile costs about 0.78 of a 256x256
        // one; it wins when the wider tile would leave much of its last round idle (narrow N).
        if (a.epilogue != kEpiSwiglu && a.M > 512) {
            const int t192 = ceil_div(a.M, 256) * ceil_div(a.N, 192);
            if (ceil_div(t192, 256) * 0.78 < ceil_div(t256, 256) * 0.97) return TileCfg{kKidGemm256x192, 256, 192};
        }
        return TileCfg{kKidGemm256, 256, 256};
    }
    if (a.K <= 4096 && a.K % kBK == 0 && a.epilogue != kEpiSwiglu && a.path != 2) {
        if (rope_direct(a)) return TileCfg{kKidGemm32, 32, 128};
        // a single row of 64x64 tiles leaves most CUs idle once K is deep enough to split
        if (a.M > 64 || a.K <= 2048 || a.ws == nullptr) return TileCfg{kKidGemm64x64, 64, 64};
    }
    if (a.M > 64) return TileCfg{kKidGemm128, 128, 128};
    return TileCfg{kKidGemm64, 64, 128};
}

// 128x128 and 64x128 tiles run a four-stage pipeline (128 / 96 KiB of LDS: one workgroup per CU)
// when the launch has at most one workgroup per CU anyway: operands that come from HBM need the
// deeper prefetch.  A deep K is split so that this holds.
bool deep_pipeline(const GemmArgs& a, const TileCfg& t) {
    if ((t.id != kKidGemm128 && t.id != kKidGemm64) || a.K % kBK != 0 || a.path == 2) return false;
    const int tiles = ceil_div(a.M, t.bm) * ceil_div(a.N, t.bn);
    return tiles <= 256 && (a.K >= 4096 || tiles >= 128 || a.ws == nullptr);
}

// How many K splits: fill the chip (>= ~256 workgroups) without making the slabs per split
// too few, and only when the workspace can hold the partials.
int pick_splits(const GemmArgs& a, const TileCfg& t) {
    if (t.id == kKidGemm32 || t.id == kKidGemm64x64) return 1;
    if ((t.id == kKidGemm256x192 || t.id == kKidGemm256x160) && a.epilogue == kEpiSwiglu) return 1;
    const int tiles = ceil_div(a.M, t.bm) * ceil_div(a.N, t.bn);
    if (tiles >= 128 || a.K < 1024) return 1;  // half a chip of tiles: splitting costs more than it gains
    // one workgroup per CU with the deep pipeline, two otherwise
    int splits = deep_pipeline(a, t) ? 256 / tiles : ceil_div(256, tiles);
    const int max_by_k = a.K / 512;  // at least 8 slabs per split
    splits = splits < max_by_k ? splits : max_by_k;
    if (splits > 16) splits = 16;
    while (splits > 1 && (size_t)splits * a.M * a.N * 4 > a.ws_bytes) --splits;
    return splits < 1 ? 1 : splits;
}

// The fused reduction + rotary kernel keeps one fp32 row in LDS and addresses C with row stride N.
bool rope_fusable(const GemmArgs& a) {
    return a.rope && a.epilogue == kEpiStore && a.ldc == a.N && a.N <= 12288 &&
           a.N == (a.rope->Hq + 2 * a.rope->Hkv) * a.rope->dh;
}

// The fused reduction + RMSNorm kernel works on 16-byte column groups.
bool norm_fusable(const GemmArgs& a) {
    return a.norm_out && a.N <= 8192 && a.N % 4 == 0 && a.ldc % 4 == 0 && ((uintptr_t)a.C % 16 == 0) &&
           ((uintptr_t)a.norm_out % 8 == 0) && ((uintptr_t)a.norm_gain % 8 == 0);
}

// What gemm_dma2_kernel needs beyond whole 64-deep slabs: at least as many slabs as stages in every K split, and
// the weight rows (from the matrix start) and a tile's activation rows within reach of a 32-bit byte offset.
bool dma2_ok(const GemmArgs& a, int splits, int stages = 2) {
    const int k_per_split = ceil_div(ceil_div(a.K, splits), kBK) * kBK;
    return a.K % kBK == 0 && a.path != 2 && k_per_split >= stages * kBK &&
           a.K - (splits - 1) * k_per_split >= stages * kBK &&
           (uint64_t)a.N * (uint64_t)a.ldw * sizeof(bf16) < (1ull << 32) &&
           (uint64_t)256 * (uint64_t)a.lda * sizeof(bf16) < (1ull << 32);  // a tile's activation rows as well
}

template <int BM, int BN, int WM, int WN, int EPI, int SWIGLU, int DST = kDmaStages, int DBK = kDmaBK>
hipError_t launch_one(const GemmArgs& a, int splits, void* out, hipStream_t s) {
    // direct-to-LDS pipeline shape: DBK-deep slabs in DST stages
    const int gm = ceil_div(a.M, BM), gn = ceil_div(a.N, BN);
    const int n_tiles = gm * gn;
    const int per_xcd = ceil_div(n_tiles * splits, kXcd);  // work items (tile, split) per XCD
    const int k_per_split = ceil_div(ceil_div(a.K, splits), kBK) * kBK;
    const dim3 grid((unsigned)(per_xcd * kXcd)), block(WM * WN * 64);
    // direct-to-LDS loads need whole 64-deep slabs; path 2 keeps the register-staged kernel
    const bool dma = a.K % kBK == 0 && a.path != 2;
    // The wide two-stage tiles run on gemm_dma2_kernel (what it does not take goes to the register-staged kernel).
    constexpr bool kWide = DST == 2 && DBK == 64 && BM >= 128 && EPI != kEpiRope;
    if constexpr (kWide) {
        // The decode gate/up tile leaves room for a third stage in the 160 KiB of LDS: two slabs in flight
        // feed a workgroup that streams its weights from HBM (measured at 512 rows, weights not cached:
        // 35.8 -> 34.3 us at K = 1536, 81.1 -> 78.8 us at K = 3584).
        constexpr int S = (BM == 256 && BN == 160) ? 3 : 2;
        if (dma2_ok(a, splits, S)) {
            const size_t lds = (size_t)S * (BM + BN) * 64 * sizeof(bf16);
            auto kern = gemm_dma2_kernel<BM, BN, WM, WN, EPI, SWIGLU, S>;
            static bool attr_set2 = false;  // one flag per template instance
            if (!attr_set2) {
                hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                if (e != hipSuccess) return e;
                attr_set2 = true;
            }
            // Many rounds of tiles: one resident workgroup per CU slot walks its share of them (no gap
            // between tiles, the next tile's first loads overlap the epilogue).  Few rounds: one tile per
            // workgroup, placed by the dispatcher.
            const int nvb = per_xcd * kXcd;
            const int resident = 256 * (lds > 80 * 1024 ? 1 : 2);
            const int g = nvb >= 4 * resident ? resident : nvb;
            kern<<<dim3((unsigned)g), block, lds, s>>>((const bf16*)a.A, a.lda, (const bf16*)a.W, a.ldw, out, a.ldc, a.M, a.N,
                                                       a.K, gm, gn, n_tiles, splits, k_per_split, a.N / 2, nvb,
                                                       (EPI == kEpiLse && a.lse) ? *a.lse
                                                       : (EPI == kEpiLogitsMax && a.block_max) ? *a.block_max : LseFuse{});
            return hipGetLastError();
        }
    } else if (dma) {
        size_t lds = (size_t)DST * (BM + BN) * DBK * sizeof(bf16);
        if (EPI == kEpiRope) {  // fp32 tile [BM][BN + 1] + per-row position and page
            const size_t need = (size_t)BM * (BN + 1) * 4 + (size_t)(BM + (BM & 1)) * 4 + (size_t)BM * 8;
            lds = lds > need ? lds : need;
        }
        auto kern = gemm_dma_kernel<BM, BN, WM, WN, EPI, SWIGLU, DBK, DST>;
        static bool attr_set = false;  // one flag per template instance
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        kern<<<grid, block, lds, s>>>((const bf16*)a.A, a.lda, (const bf16*)a.W, a.ldw, out, a.ldc, a.M, a.N, a.K,
                                      gm, gn, n_tiles, splits, k_per_split, a.N / 2,
                                      (EPI == kEpiRope && a.rope) ? *a.rope : RopeKvArgs{}, LseFuse{});
        return hipGetLastError();
    }
    if constexpr (EPI == kEpiRope || EPI == kEpiLse || EPI == kEpiLogitsMax) {
        return hipErrorInvalidValue;  // only the direct-to-LDS kernel has this epilogue
    } else {
        const size_t lds = (size_t)2 * (BM + BN) * kLdsRow * sizeof(bf16);
        auto kern = gemm_mfma_kernel<BM, BN, WM, WN, EPI, SWIGLU>;
        static bool attr_set = false;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        kern<<<grid, block, lds, s>>>((const bf16*)a.A, a.lda, (const bf16*)a.W, a.ldw, out, a.ldc, a.M, a.N, a.K,
                                      gm, gn, n_tiles, splits, k_per_split, a.N / 2);
        return hipGetLastError();
    }
}

template <int BM, int BN, int WM, int WN, int DST = kDmaStages, int DBK = kDmaBK>
hipError_t launch_tile(const GemmArgs& a, int splits, hipStream_t s) {
    const bool sw = a.epilogue == kEpiSwiglu;
    constexpr bool kPairs = (BN / WN / 32) % 2 == 0;  // a wave holds gate/up block pairs
    if (sw && !kPairs) return hipErrorInvalidValue;
    if (splits > 1) {
        hipError_t e;
        if constexpr (kPairs) {
            e = sw ? launch_one<BM, BN, WM, WN, kEpiPartial, true, DST, DBK>(a, splits, a.ws, s)
                   : launch_one<BM, BN, WM, WN, kEpiPartial, false, DST, DBK>(a, splits, a.ws, s);
        } else {
            e = launch_one<BM, BN, WM, WN, kEpiPartial, false, DST, DBK>(a, splits, a.ws, s);
        }
        if (e != hipSuccess) return e;
        const int64_t n_out = sw ? (int64_t)a.M * (a.N / 2) : (int64_t)a.M * a.N;
        const unsigned blocks = (unsigned)ceil_div64(n_out, 256);
        const float* P = (const float*)a.ws;
        switch (a.epilogue) {
            case kEpiStore:
                if (rope_fusable(a)) {
                    gemm_splitk_reduce_rope_kernel<<<a.M, 256, (size_t)a.N * 4, s>>>(P, splits, a.M, a.N, *a.rope);
                    return hipGetLastError();
                }
                gemm_splitk_reduce_kernel<kEpiStore><<<blocks, 256, 0, s>>>(P, splits, a.M, a.N, a.C, a.ldc);
                break;
            case kEpiStoreF32:
                gemm_splitk_reduce_kernel<kEpiStoreF32><<<blocks, 256, 0, s>>>(P, splits, a.M, a.N, a.C, a.ldc);
                break;
            case kEpiAddF32:
                if (norm_fusable(a)) {
                    gemm_splitk_reduce_norm_kernel<<<a.M, 256, 0, s>>>(P, splits, a.M, a.N, (float*)a.C, a.ldc,
                                                                        (const bf16*)a.norm_gain, a.norm_eps,
                                                                        (bf16*)a.norm_out);
                    return hipGetLastError();
                }
                gemm_splitk_reduce_kernel<kEpiAddF32><<<blocks, 256, 0, s>>>(P, splits, a.M, a.N, a.C, a.ldc);
                break;
            default:
                gemm_splitk_reduce_kernel<kEpiSwiglu><<<blocks, 256, 0, s>>>(P, splits, a.M, a.N, a.C, a.ldc);
                break;
        }
        return hipGetLastError();
    }
    switch (a.epilogue) {
        case kEpiStore:
            return launch_one<BM, BN, WM, WN, kEpiStore, false, DST, DBK>(a, 1, a.C, s);
        case kEpiStoreF32:
            return launch_one<BM, BN, WM, WN, kEpiStoreF32, false, DST, DBK>(a, 1, a.C, s);
        case kEpiAddF32:
            return launch_one<BM, BN, WM, WN, kEpiAddF32, false, DST, DBK>(a, 1, a.C, s);
        case kEpiSwiglu:
            if constexpr (kPairs) return launch_one<BM, BN, WM, WN, kEpiSwiglu, true, DST, DBK>(a, 1, a.C, s);
            return hipErrorInvalidValue;
        default:
            return hipErrorInvalidValue;
    }
}

template <typename T>
hipError_t launch_generic(const GemmArgs& a, hipStream_t s) {
    if (a.epilogue == kEpiSwiglu) {
        const int F = a.N / 2;
        gemm_generic_swiglu_kernel<T><<<dim3(ceil_div(F, 256), a.M), 256, 0, s>>>(
            (const T*)a.A, a.lda, (const T*)a.W, a.ldw, (T*)a.C, a.ldc, a.M, F, a.K);
        return hipGetLastError();
    }
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

}  // namespace

int gemm_fuses_lse(const GemmArgs& a) {
    if (a.epilogue != kEpiStoreF32 || !mfma_ok(a) || !dma2_ok(a, 1)) return 0;
    if (pick_tile(a).id != kKidGemm256) return 0;
    return ceil_div(a.N, 256) * 4;  // one block per wave column of a 256-wide tile
}

int gemm_fuses_max(const GemmArgs& a) {
    if (gemm_fuses_lse(a) == 0) return 0;  // same kernel shape
    // the transposed epilogue stores 16-byte column quads
    if (a.N % 4 != 0 || a.ldc % 4 != 0 || (uintptr_t)a.C % 16 != 0) return 0;
    return ceil_div(a.N, 256) * 4;
}

size_t gemm_splitk_scratch_bytes(const GemmArgs& a) {
    if (!mfma_ok(a) || a.M <= 0 || a.N <= 0) return 0;
    GemmArgs u = a;
    u.ws = (void*)(uintptr_t)256;  // never dereferenced: only "a workspace exists"
    u.ws_bytes = ~(size_t)0;
    const int splits = pick_splits(u, pick_tile(u));
    return splits > 1 ? (size_t)splits * a.M * a.N * sizeof(float) : 0;
}

int gemm_kernel_id(const GemmArgs& a) {
    if (!mfma_ok(a)) return kKidGemmGeneric;
    const int id = pick_tile(a).id;
    // the heaviest instantiation of a rollout step is reported on its own
    return (id == kKidGemm256 && a.epilogue == kEpiSwiglu) ? (int)kKidGemm256Swiglu : id;
}

static hipError_t launch_gemm_only(const GemmArgs& a, int splits, const TileCfg& t, hipStream_t s) {
    switch (t.id) {
        case kKidGemm256:
            return launch_tile<256, 256, 2, 4>(a, splits, s);
        case kKidGemm128:
            if (deep_pipeline(a, t)) return launch_tile<128, 128, 2, 2, 4>(a, splits, s);
            return launch_tile<128, 128, 2, 2>(a, splits, s);
        case kKidGemm32:
            if (rope_direct(a)) {
                // one round of workgroups: 64-row tiles once the 32-row ones outnumber the CUs
                if (ceil_div(a.M, 32) * (a.N / 128) > 256) return launch_one<64, 128, 1, 4, kEpiRope, 0, 4>(a, 1, a.C, s);
                return launch_one<32, 128, 1, 4, kEpiRope, 0, 4>(a, 1, a.C, s);
            }
            return launch_tile<32, 128, 1, 4, 4>(a, splits, s);
        case kKidGemm64x64:
            return launch_tile<64, 64, 2, 2, 4>(a, splits, s);
        case kKidGemm256x160:
            return launch_one<256, 160, 4, 1, kEpiSwiglu, 2>(a, 1, a.C, s);
        case kKidGemm256x192:
            if (a.epilogue == kEpiSwiglu) return launch_one<256, 192, 4, 2, kEpiSwiglu, 2>(a, 1, a.C, s);
            return launch_tile<256, 192, 4, 2>(a, splits, s);
        default:
            if (deep_pipeline(a, t)) return launch_tile<64, 128, 1, 2, 4>(a, splits, s);
            // up to two workgroups per CU: three stages (72 KiB each) still fit twice
            if (a.K % kBK == 0 && a.path != 2 && ceil_div(a.M, 64) * ceil_div(a.N, 128) * splits <= 512)
                return launch_tile<64, 128, 1, 2, 3>(a, splits, s);
            return launch_tile<64, 128, 1, 2>(a, splits, s);
    }
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    const bool want_norm = a.norm_out != nullptr && a.epilogue == kEpiAddF32;
    hipError_t e;
    bool norm_done = false, rope_done = false;
    if (!mfma_ok(a)) {
        e = a.dtype == kF32 ? launch_generic<float>(a, s) : launch_generic<bf16>(a, s);
    } else {
        const TileCfg t = pick_tile(a);
        const int splits = (a.ws && a.ws_bytes) ? pick_splits(a, t) : 1;
        if (a.lse && gemm_fuses_lse(a) > 0) {
            a.lse->blocks = gemm_fuses_lse(a);
            return launch_one<256, 256, 2, 4, kEpiLse, false>(a, 1, nullptr, s);
        }
        if (a.block_max && gemm_fuses_max(a) > 0) {
            a.block_max->blocks = gemm_fuses_max(a);
            return launch_one<256, 256, 2, 4, kEpiLogitsMax, false>(a, 1, a.C, s);
        }
        e = launch_gemm_only(a, splits, t, s);
        norm_done = want_norm && splits > 1 && norm_fusable(a);  // fused into the K-split reduction
        rope_done = (splits > 1 && rope_fusable(a)) || (t.id == kKidGemm32 && rope_direct(a));
    }
    if (e != hipSuccess) return e;
    if (a.rope && a.epilogue == kEpiStore && !rope_done) return launch_rope_kv(*a.rope, s);
    if (!want_norm || norm_done) return e;
    return launch_rmsnorm((const float*)a.C, nullptr, a.norm_gain, a.dtype, a.N, a.norm_eps, a.norm_out, a.M, s);
}

}  // namespace rpo
