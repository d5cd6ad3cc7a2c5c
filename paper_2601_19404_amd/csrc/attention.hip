// Causal grouped-query attention over the paged KV cache.
//
//  * attn_generic_kernel: one wave per (row, query head), fp32 math on the vector
//    ALUs, any dtype / head_dim <= 256 / page size.  Used by the fp32 tiny model.
//  * MFMA kernels (bf16, head_dim 128, 64-token pages): a workgroup of four waves
//    holds up to 64 query rows (16 per wave) in registers and streams KV pages
//    through LDS, double buffered.  Scores are computed TRANSPOSED,
//    S^T = K Q^T (v_mfma_f32_16x16x32_bf16: K rows are the A operand, query rows the
//    B operand), so each lane owns one query row's scores: the online-softmax
//    statistics are per lane, and the probabilities already sit in the B-operand
//    layout of the second product O^T = V^T P^T (V pages are stored transposed).
//      - attn_chunk_mfma_kernel: prefill / teacher-forced chunks; a tile packs
//        floor(64 / (Hq/Hkv)) consecutive positions x the query heads of one KV head.
//      - attn_decode_mfma_kernel: one new query per rollout.  The rollouts of a
//        group share their prefix pages (RPO Sec. 3.4: the sampling group shares the
//        response prefix), so ONE workgroup multiplies each shared page with the
//        G * (Hq/Hkv) query rows of the whole group: the prefix is read from HBM once
//        per group, not once per rollout.  Private suffix pages are handled per
//        rollout; pieces are merged by log-sum-exp (attn_merge_kernel).
#include "kernels.hpp"

namespace rpo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// generic kernel
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(64) void attn_generic_kernel(AttnArgs a) {
    __shared__ float qs[256];
    __shared__ float ps[64];
    const int r = blockIdx.x, hq = blockIdx.y, lane = threadIdx.x;
    if (a.active && !a.active[r]) return;
    const int seq = a.row_seq ? a.row_seq[r] : r;
    if (seq < 0) return;  // padding row of a compacted batch
    const SeqDesc sd = a.seqs[seq];
    const int ctx = sd.pos0 + (a.single_row ? 0 : r - sd.row_start) + a.pos_add + 1;
    const int kh = hq / (a.Hq / a.Hkv);
    const int dh = a.dh, pt = a.geom.page_tokens;
    const T* q = (const T*)a.q + (int64_t)r * a.q_stride + (int64_t)hq * dh;
    for (int d = lane; d < dh; d += 64) qs[d] = to_f32<T>(q[d]);
    __syncthreads();
    const T* pool = (const T*)a.kv_pool;
    const int32_t* table = a.tables + sd.table_off;
    float o[4] = {0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;
    for (int c0 = 0; c0 < ctx; c0 += 64) {
        const int tok = c0 + lane;
        float s = -INFINITY;
        int page = 0;
        if (tok < ctx) {
            page = table[tok / pt];
            const T* kp = pool + a.geom.k_block(a.layer, page, kh) + (int64_t)(tok % pt) * dh;
            float dot = 0.f;
            for (int d = 0; d < dh; ++d) dot = fmaf(qs[d], to_f32<T>(kp[d]), dot);
            s = dot * a.scale;
        }
        const float mnew = fmaxf(m, wave_max(s));  // finite: token c0 is always visible
        const float p = (tok < ctx) ? expf(s - mnew) : 0.f;
        const float alpha = expf(m - mnew);
        l = l * alpha + wave_sum(p);
        m = mnew;
        __syncthreads();
        ps[lane] = p;
        __syncthreads();
        const int nt = min(64, ctx - c0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int d = lane + 64 * i;
            float acc = o[i] * alpha;
            for (int t = 0; t < nt; ++t) {
                const int pg = __shfl(page, t, 64);
                if (d < dh) {
                    const int slot = (c0 + t) % pt;
                    acc = fmaf(ps[t], to_f32<T>(pool[a.geom.v_block(a.layer, pg, kh) + a.geom.v_elem(slot, d)]),
                               acc);
                }
            }
            o[i] = acc;
        }
    }
    T* out = (T*)a.out + (int64_t)r * a.Hq * dh + (int64_t)hq * dh;
    const float inv = 1.0f / l;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int d = lane + 64 * i;
        if (d < dh) out[d] = from_f32<T>(o[i] * inv);
    }
}

static hipError_t launch_attn_generic(const AttnArgs& a, hipStream_t s) {
    const dim3 grid(a.rows, a.Hq);
    if (a.dtype == kF32)
        attn_generic_kernel<float><<<grid, 64, 0, s>>>(a);
    else
        attn_generic_kernel<bf16><<<grid, 64, 0, s>>>(a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// MFMA core
// ---------------------------------------------------------------------------
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
constexpr int kDh = 128;      // head_dim of the MFMA kernels
constexpr int kPt = 64;       // tokens per page
// LDS tiles are unpadded; bank conflicts of the fragment reads are avoided by permuting the 16-byte
// pieces of a row with the row index.  K tile [64 tokens][128 channels]: piece p of row r sits at
// p ^ (r & 15), so the 16-byte reads of sixteen consecutive rows (same piece) are spread evenly
// over the banks whichever lanes the LDS serves together.
// V^T tile [128 channels][64 tokens]: inside a row the tokens are reordered so that the eight tokens a
// lane group multiplies in one k-step of the second product (32 kk + 4 g + i and 32 kk + 16 + 4 g + i,
// i < 4: the token order its probabilities leave the first product in) are one 16-byte piece, piece
// 4 kk + g; piece p of row r sits at p ^ (r & 7) ^ ((r >> 3) & 1), which spreads the 16-byte reads of
// sixteen consecutive rows (same piece) over the banks.
constexpr int kKRow = kDh;  // LDS row of the K tile  [64][128]
constexpr int kVRow = kPt;  // LDS row of the V^T tile [128][64]
constexpr int kKTile = kPt * kKRow;
constexpr int kVTile = kDh * kVRow;
constexpr size_t kAttnLds = (size_t)2 * (kKTile + kVTile) * sizeof(bf16);

// Maximum over the four lanes l % 16, l % 16 + 16, + 32, + 48 (the lanes that share a query column), in
// every one of them.  The two lane-swap instructions of gfx950 exchange rows of 16 (halves of 32) lanes
// between two registers: fed the same value twice, they leave in every lane its own value and that of
// lane ^ 16 (lane ^ 32) -- a register exchange, no trip through LDS as a general shuffle takes.
__device__ inline float max_over_lane_groups(float v) {
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// NC = 16-column query tiles per wave: a wave multiplies every K / V fragment it reads from LDS
// with NC query tiles, so the LDS traffic per flop falls with NC.
template <int NC>
struct AttnState {
    f32x4_t ot[NC][8];  // O^T: lane = query column (lane % 16), rows 16 * mb + 4 * (lane / 16) + i
    float m[NC], l[NC];  // running max (raw scores inside the loop, log2 domain on return) and this lane's share of the running sum
};

// Stream pages [page_begin, page_end) of `table` against this lane's NC query rows.
//   qptr[c]  : the lane's query row (128 bf16) of column tile c, or nullptr for a padding column
//   limit[c] : tokens visible to that query (absolute count; 0 for padding)
// Must be called by all 256 threads with the same page range.
template <int NC>
__device__ inline void attn_stream_pages(const bf16* const (&qptr)[NC], const int (&limit)[NC], const bf16* pool,
                                         const KvGeom& geom, int layer, int kh, const int32_t* table,
                                         int page_begin, int page_end, float scale_log2, bf16* smem,
                                         bool wave_live, AttnState<NC>& st) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int c16 = lane & 15, g = lane >> 4;
    bf16* Ks = smem;                 // [2][kKTile]
    bf16* Vs = smem + 2 * kKTile;    // [2][kVTile]

#pragma unroll
    for (int c = 0; c < NC; ++c) {
#pragma unroll
        for (int i = 0; i < 8; ++i) st.ot[c][i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        st.m[c] = -INFINITY;
        st.l[c] = 0.f;
    }
    const int np = page_end - page_begin;
    if (np <= 0) return;

    bf16x8_t bq[NC][4];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (qptr[c])
                bq[c][kk] = *(const bf16x8_t*)(qptr[c] + kk * 32 + 8 * g);
            else
#pragma unroll
                for (int e = 0; e < 8; ++e) bq[c][kk][e] = (__bf16)0.0f;
        }

    // smallest visible-token count among this wave's real queries (padding columns never mask)
    int lim_min = 0x7fffffff;
#pragma unroll
    for (int c = 0; c < NC; ++c)
        if (qptr[c]) lim_min = min(lim_min, limit[c]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lim_min = min(lim_min, __shfl_xor(lim_min, o, 64));

    const f32x4_t zero4 = f32x4_t{0.f, 0.f, 0.f, 0.f};
    u32x4_t rk[4], rv[4];
    auto load_page = [&](int p) {
        const int64_t page = table[p];
        const u32x4_t* kb = (const u32x4_t*)(pool + geom.k_block(layer, page, kh));
        const u32x4_t* vb = (const u32x4_t*)(pool + geom.v_block(layer, page, kh));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            rk[i] = kb[tid + i * 256];
            rv[i] = vb[tid + i * 256];
        }
    };
    auto store_page = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * 256;
            const int kr = c >> 4;
            *(u32x4_t*)(Ks + buf * kKTile + kr * kKRow + (((c & 15) ^ (kr & 15)) << 3)) = rk[i];
            // V block piece c = (token group m = c / 128: tokens 8 m .. 8 m + 7, channel c % 128) -> LDS row =
            // channel; tokens 8 m .. + 3 are half (m / 2) % 2 of piece 4 (m / 4) + (2 m) % 4, tokens 8 m + 4 .. + 7
            // the same half of the piece after it
            const int vr = c & (kDh - 1), m = c >> 7;
            const int sw = (vr & 7) ^ ((vr >> 3) & 1);
            const int pl = 4 * (m >> 2) + ((2 * m) & 3);
            bf16* vrow = Vs + buf * kVTile + vr * kVRow + 4 * ((m >> 1) & 1);
            *(u32x2_t*)(vrow + ((pl ^ sw) << 3)) = u32x2_t{rv[i].x, rv[i].y};
            *(u32x2_t*)(vrow + (((pl + 1) ^ sw) << 3)) = u32x2_t{rv[i].z, rv[i].w};
        }
    };

    load_page(page_begin);
    store_page(0);
    __syncthreads();
    for (int p = 0; p < np; ++p) {
        const int buf = p & 1;
        if (p + 1 < np) load_page(page_begin + p + 1);
        if (wave_live) {
            const bf16* ks = Ks + buf * kKTile;
            const bf16* vs = Vs + buf * kVTile;
            const int tok0 = (page_begin + p) * kPt;
            f32x4_t sc[NC][4];
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const bf16x8_t ak = *(const bf16x8_t*)(ks + (mb * 16 + c16) * kKRow + (((kk * 4 + g) ^ c16) << 3));
#pragma unroll
                    for (int c = 0; c < NC; ++c)  // the first product starts from one shared zero block
                        sc[c][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ak, bq[c][kk], kk == 0 ? zero4 : sc[c][mb], 0, 0, 0);
                }
            }
            bf16x8_t bp[NC][2];
            const bool need_mask = tok0 + kPt > lim_min;  // wave-uniform: some query here does not see the whole page
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                // online softmax in the raw score domain: p = 2^((s - m) * scale_log2)
                float mloc = -INFINITY;
                if (need_mask) {
#pragma unroll
                    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int tok = tok0 + mb * 16 + 4 * g + i;
                            const float s = (tok < limit[c]) ? sc[c][mb][i] : -INFINITY;
                            sc[c][mb][i] = s;
                            mloc = fmaxf(mloc, s);
                        }
                } else {
#pragma unroll
                    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                        for (int i = 0; i < 4; ++i) mloc = fmaxf(mloc, sc[c][mb][i]);
                }
                mloc = max_over_lane_groups(mloc);
                const float mnew = fmaxf(st.m[c], mloc);
                const float muse = (mnew == -INFINITY) ? 0.f : mnew;
                const float alpha = __builtin_amdgcn_exp2f((st.m[c] - muse) * scale_log2);
                const float nb = -muse * scale_log2;
                float lsum = 0.f;
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[c][mb][i], scale_log2, nb));
                        sc[c][mb][i] = pv;
                        lsum += pv;
                    }
                st.l[c] = st.l[c] * alpha + lsum;
                st.m[c] = mnew;
                if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {  // the running maximum moved in some lane
#pragma unroll
                    for (int mb2 = 0; mb2 < 8; ++mb2) st.ot[c][mb2] *= alpha;
                }
                // K slot (g, j) of the second product <-> token 32 kk2 + 4 g + j      (j < 4)
                //                                     token 32 kk2 + 16 + 4 g + j - 4 (j >= 4)
#pragma unroll
                for (int kk2 = 0; kk2 < 2; ++kk2)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        bp[c][kk2][i] = (__bf16)sc[c][2 * kk2][i];
                        bp[c][kk2][4 + i] = (__bf16)sc[c][2 * kk2 + 1][i];
                    }
            }
#pragma unroll
            for (int kk2 = 0; kk2 < 2; ++kk2) {
#pragma unroll
                for (int mb2 = 0; mb2 < 8; ++mb2) {
                    const bf16x8_t av = *(const bf16x8_t*)(vs + (mb2 * 16 + c16) * kVRow +
                                                           (((4 * kk2 + g) ^ (c16 & 7) ^ (c16 >> 3)) << 3));
#pragma unroll
                    for (int c = 0; c < NC; ++c)
                        st.ot[c][mb2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bp[c][kk2], st.ot[c][mb2], 0, 0, 0);
                }
            }
        }
        if (p + 1 < np) store_page(buf ^ 1);
        __syncthreads();
    }
    // every lane of a query column ends with the full row sum; the maximum leaves in the log2 domain
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        st.l[c] += __shfl_xor(st.l[c], 16, 64);
        st.l[c] += __shfl_xor(st.l[c], 32, 64);
        st.m[c] *= scale_log2;
    }
}

// ---------------------------------------------------------------------------
// chunk kernel: grid (q tile, kv head, sequence)
// ---------------------------------------------------------------------------
constexpr int kChunkNC = 2;                  // 16-column query tiles per wave of the chunk kernel
constexpr int kChunkCols = 64 * kChunkNC;   // query columns (position x head) per workgroup

__global__ __launch_bounds__(256, 2) void attn_chunk_mfma_kernel(AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const SeqDesc sd = a.seqs[blockIdx.z];
    const int hpk = a.Hq / a.Hkv;
    const int ntt = kChunkCols / hpk;  // positions per tile
    const int n_tiles = (sd.n_rows + ntt - 1) / ntt;
    if ((int)blockIdx.x >= n_tiles) return;
    const int qt = n_tiles - 1 - blockIdx.x;  // longest contexts first
    const int kh = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bf16* qptr[kChunkNC];
    int limit[kChunkNC], head[kChunkNC];
    int64_t row[kChunkNC];
#pragma unroll
    for (int c = 0; c < kChunkNC; ++c) {
        const int col = (wave * kChunkNC + c) * 16 + (lane & 15);
        const int tl = qt * ntt + col / hpk;  // row of the sequence
        const bool valid = col < ntt * hpk && tl < sd.n_rows;
        head[c] = kh * hpk + col % hpk;
        row[c] = sd.row_start + tl;
        qptr[c] = valid ? (const bf16*)a.q + row[c] * a.q_stride + (int64_t)head[c] * kDh : nullptr;
        limit[c] = valid ? sd.pos0 + tl + a.pos_add + 1 : 0;
    }
    const int last_tl = min(sd.n_rows, (qt + 1) * ntt) - 1;
    const int max_limit = sd.pos0 + last_tl + a.pos_add + 1;
    const int first_col_of_wave = wave * kChunkNC * 16;
    const bool wave_live = first_col_of_wave < ntt * hpk && qt * ntt + first_col_of_wave / hpk < sd.n_rows;

    AttnState<kChunkNC> st;
    attn_stream_pages<kChunkNC>(qptr, limit, (const bf16*)a.kv_pool, a.geom, a.layer, kh, a.tables + sd.table_off, 0,
                                (max_limit + kPt - 1) / kPt, a.scale * 1.4426950408889634f, (bf16*)smem_raw,
                                wave_live, st);
    const int g = lane >> 4;
#pragma unroll
    for (int c = 0; c < kChunkNC; ++c) {
        if (!qptr[c]) continue;
        const float inv = 1.0f / st.l[c];
        bf16* out = (bf16*)a.out + row[c] * (int64_t)a.Hq * kDh + (int64_t)head[c] * kDh;
#pragma unroll
        for (int mb2 = 0; mb2 < 8; ++mb2) {
            bf16x4_t o4;
#pragma unroll
            for (int i = 0; i < 4; ++i) o4[i] = (__bf16)(st.ot[c][mb2][i] * inv);
            *(bf16x4_t*)(out + mb2 * 16 + 4 * g) = o4;
        }
    }
}

// ---------------------------------------------------------------------------
// decode kernel: grid (part, kv head, group)
//   part <  n_split * n_ct : shared-prefix piece `split` for column tile `ct`
//   part >= n_split * n_ct : private pages of rollout (part - n_split * n_ct) of the group
// Partials per (rollout row, query head): n_split + 1 pieces of (m, l, O[128]).
// ---------------------------------------------------------------------------
struct DecodeGeom {
    int G, n_split, n_ct, rpt;  // rollouts per column tile
    int n_rows;                 // rollout rows covered (r = group * G + i < n_rows)
    const int32_t* row_of;      // compacted batch: rollout -> query / output row (< 0: finished), or NULL
};

__global__ __launch_bounds__(256) void attn_decode_mfma_kernel(AttnArgs a, DecodeGeom dg,
                                                               const int32_t* __restrict__ shared_pages,
                                                               float* __restrict__ part_o,
                                                               float* __restrict__ part_ml) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const int grp = blockIdx.z, kh = blockIdx.y, part = blockIdx.x;
    const int hpk = a.Hq / a.Hkv;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = wave * 16 + (lane & 15);
    const int n_shared = shared_pages[grp];
    const int n_pref = dg.n_split * dg.n_ct;

    // Uniform per workgroup: whose page table is walked (trow) and which pages.
    // Per lane: which rollout / head the lane's query column belongs to.
    int ri, piece, page_begin, page_end, trow;
    bool col_ok, wave_live;
    if (part < n_pref) {
        const int split = part % dg.n_split, ct = part / dg.n_split;
        ri = ct * dg.rpt + col / hpk;
        col_ok = col < dg.rpt * hpk && ri < dg.G;
        const int first = wave * 16;
        wave_live = first < dg.rpt * hpk && ct * dg.rpt + first / hpk < dg.G;
        const int pps = (n_shared + dg.n_split - 1) / dg.n_split;
        page_begin = min(n_shared, split * pps);
        page_end = min(n_shared, page_begin + pps);
        piece = split;
        trow = grp * dg.G;  // any rollout of the group: their first n_shared table entries agree
    } else {
        ri = part - n_pref;
        col_ok = col < hpk;
        wave_live = wave * 16 < hpk;  // up to 64 query heads per KV head: one 16-column tile per wave
        page_begin = n_shared;
        page_end = n_shared;  // extended below if the rollout is alive
        piece = dg.n_split;
        trow = grp * dg.G + ri;
    }
    // a rollout is live if it has a query row: its row in a compacted batch, else its active flag
    auto query_row = [&](int rollout) -> int {
        if (rollout >= dg.n_rows) return -1;
        if (dg.row_of) return dg.row_of[rollout];
        return (a.active && !a.active[rollout]) ? -1 : rollout;
    };
    const bool trow_ok = trow < dg.n_rows;
    const SeqDesc sd = a.seqs[trow_ok ? trow : 0];
    const int ctx = sd.pos0 + a.pos_add + 1;  // the same for every rollout of a group
    if (part >= n_pref && query_row(trow) >= 0) page_end = (ctx + kPt - 1) / kPt;
    if (!trow_ok) page_end = page_begin;
    const int row = grp * dg.G + ri;          // rollout
    const int qrow = col_ok ? query_row(row) : -1;
    const bool valid = qrow >= 0;
    const int head = kh * hpk + col % hpk;
    const bf16* const qptr[1] = {valid ? (const bf16*)a.q + (int64_t)qrow * a.q_stride + (int64_t)head * kDh : nullptr};
    const int limit[1] = {valid ? ctx : 0};

    AttnState<1> st;
    attn_stream_pages<1>(qptr, limit, (const bf16*)a.kv_pool, a.geom, a.layer, kh, a.tables + sd.table_off,
                         page_begin, page_end, a.scale * 1.4426950408889634f, (bf16*)smem_raw, wave_live, st);
    if (!valid) return;
    const int g = lane >> 4;
    const int64_t slot = ((int64_t)row * a.Hq + head) * (dg.n_split + 1) + piece;
    float* po = part_o + slot * kDh;
#pragma unroll
    for (int mb2 = 0; mb2 < 8; ++mb2) *(f32x4_t*)(po + mb2 * 16 + 4 * g) = st.ot[0][mb2];
    if (g == 0) {
        part_ml[2 * slot] = st.m[0];
        part_ml[2 * slot + 1] = st.l[0];
    }
}

// One workgroup per rollout row, one thread per (query head, pair of output channels): combine
// the pieces.  All loads of a thread are issued before any is used (at most kMaxPieces pieces).
constexpr int kMaxPieces = 9;  // decode_splits() caps the prefix pieces at 8, plus the private one
// Query row blockIdx.x belongs to rollout row_seq[blockIdx.x] (compacted batch; < 0: padding) or to
// the rollout of the same index; the pieces are stored by rollout.
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ part_o,
                                                         const float* __restrict__ part_ml, int n_pieces,
                                                         int Hq, const uint8_t* __restrict__ active,
                                                         const int32_t* __restrict__ row_seq,
                                                         bf16* __restrict__ out) {
    const int qrow = blockIdx.x;
    const int row = row_seq ? row_seq[qrow] : qrow;
    if (row < 0 || (!row_seq && active && !active[row])) return;
    for (int w = threadIdx.x; w < Hq * (kDh / 2); w += 256) {
        const int head = w / (kDh / 2), c = (w % (kDh / 2)) * 2;
        const int64_t base = ((int64_t)row * Hq + head) * n_pieces;
        float m[kMaxPieces], l[kMaxPieces];
        float2 o[kMaxPieces];
#pragma unroll
        for (int p = 0; p < kMaxPieces; ++p) {
            const bool on = p < n_pieces;
            m[p] = on ? part_ml[2 * (base + p)] : -INFINITY;
            l[p] = on ? part_ml[2 * (base + p) + 1] : 0.f;
            o[p] = on ? *(const float2*)(part_o + (base + p) * kDh + c) : float2{0.f, 0.f};
        }
        float mx = -INFINITY;
#pragma unroll
        for (int p = 0; p < kMaxPieces; ++p) mx = fmaxf(mx, m[p]);
        float lsum = 0.f, o0 = 0.f, o1 = 0.f;
#pragma unroll
        for (int p = 0; p < kMaxPieces; ++p) {
            const float wgt = m[p] == -INFINITY ? 0.f : exp2f(m[p] - mx);  // an empty piece has no weight
            lsum += wgt * l[p];
            o0 += wgt * o[p].x;
            o1 += wgt * o[p].y;
        }
        const float inv = 1.0f / lsum;
        bf16* dst = out + ((int64_t)qrow * Hq + head) * kDh + c;
        dst[0] = f32_to_bf16(o0 * inv);
        dst[1] = f32_to_bf16(o1 * inv);
    }
}

static bool mfma_attn_ok(const AttnArgs& a) {
    const int hpk = a.Hkv > 0 ? a.Hq / a.Hkv : 0;
    return a.path != 1 && a.dtype == kBF16 && a.dh == kDh && a.geom.page_tokens == kPt && hpk >= 1 &&
           hpk <= 64 && a.q_stride % 8 == 0 && ((uintptr_t)a.q % 16 == 0);
}

bool attn_uses_mfma(const AttnArgs& a) { return mfma_attn_ok(a); }

// Raise the dynamic-LDS limit of a kernel once per process (the call is a host round trip).
static hipError_t set_attn_lds(const void* fn, bool* done) {
    if (*done) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAttnLds);
    if (e == hipSuccess) *done = true;
    return e;
}

hipError_t launch_attn_chunk(const AttnArgs& a, hipStream_t s) {
    if (a.rows <= 0 || a.n_seqs <= 0) return hipSuccess;
    if (!mfma_attn_ok(a)) return launch_attn_generic(a, s);
    static bool lds_set = false;
    hipError_t e = set_attn_lds((const void*)attn_chunk_mfma_kernel, &lds_set);
    if (e != hipSuccess) return e;
    const int ntt = kChunkCols / (a.Hq / a.Hkv);
    const dim3 grid(ceil_div(a.max_seq_rows, ntt), a.Hkv, a.n_seqs);
    attn_chunk_mfma_kernel<<<grid, 256, kAttnLds, s>>>(a);
    return hipGetLastError();
}

static int decode_splits(int n_groups_live, int Hkv, int n_ct, int max_shared_pages) {
    if (max_shared_pages <= 0) return 1;
    int want = ceil_div(512, n_groups_live * Hkv * n_ct);
    want = want < 1 ? 1 : (want > 8 ? 8 : want);
    const int cap = max_shared_pages / 2 > 0 ? max_shared_pages / 2 : 1;  // at least two pages per piece
    return want < cap ? want : cap;
}

size_t attn_decode_partial_floats(int rows, int Hq, int dh, int max_shared_pages) {
    (void)max_shared_pages;
    return (size_t)rows * Hq * 17 * (dh + 2);
}

hipError_t launch_attn_decode(const DecodeAttnArgs& d, hipStream_t s) {
    const AttnArgs& a = d.base;
    if (a.rows <= 0) return hipSuccess;
    if (!mfma_attn_ok(a)) return launch_attn_generic(a, s);
    const int hpk = a.Hq / a.Hkv;
    DecodeGeom dg;
    dg.G = d.G;
    dg.rpt = 64 / hpk < d.G ? 64 / hpk : d.G;
    dg.n_ct = ceil_div(d.G, dg.rpt);
    dg.n_rows = d.n_rollouts;
    dg.row_of = d.row_of;
    const int n_groups_live = ceil_div(d.n_rollouts, d.G);
    dg.n_split = decode_splits(n_groups_live, a.Hkv, dg.n_ct, d.max_shared_pages);
    const size_t n_slots = (size_t)d.n_rollouts * a.Hq * (dg.n_split + 1);
    if (n_slots * (kDh + 2) > d.partial_floats) return hipErrorInvalidValue;
    float* part_o = d.partial;
    float* part_ml = d.partial + n_slots * kDh;
    static bool lds_set = false;
    hipError_t e = set_attn_lds((const void*)attn_decode_mfma_kernel, &lds_set);
    if (e != hipSuccess) return e;
    const dim3 grid(dg.n_split * dg.n_ct + d.G, a.Hkv, n_groups_live);
    attn_decode_mfma_kernel<<<grid, 256, kAttnLds, s>>>(a, dg, d.shared_pages, part_o, part_ml);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (dg.n_split + 1 > kMaxPieces) return hipErrorInvalidValue;
    attn_merge_kernel<<<a.rows, 256, 0, s>>>(part_o, part_ml, dg.n_split + 1, a.Hq, a.active,
                                             d.row_of ? a.row_seq : nullptr, (bf16*)a.out);
    return hipGetLastError();
}

}  // namespace rpo
