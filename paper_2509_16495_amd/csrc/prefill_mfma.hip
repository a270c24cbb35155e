// Causal prefill attention of the local head shard over the paged KV cache (Algorithm 1, boxed
// attention line, prefill rows; chunked prefill continues a cached context).  bf16 tensors, fp32
// accumulation, head_dim 128.
//
// Tiling.  A workgroup of four wavefronts owns a tile of 128*NQB "columns"; a column is one
// (new token, query head) pair.  The query heads that share a KV head are stacked next to each
// other in the column index (GS heads per token), so one K/V tile in LDS serves the whole GQA group
// and the causal diagonal of a tile spans only 128*NQB/GS tokens.  Each wavefront owns NQB blocks
// of 32 columns and walks the keys in tiles of 64 tokens (four cache blocks):
//
//   S^T[key][col]  = K[key][:] . Q^T[:][col]          32x32x16 bf16 MFMA, A = K rows from LDS,
//                                                      B = Q^T held in registers for the whole tile
//   online softmax down each column: a lane holds 32 keys of one column in its accumulator
//   registers, the other 32 sit in lane+32, so the column max costs one cross-lane exchange
//   O^T[d][col]   += V^T[d][key] . P^T[key][col]       A = V^T rows from LDS, B = P^T taken straight
//                                                      from the softmax registers
//
// Computing the transposed products keeps P in registers: the accumulator layout of S^T (a lane
// owns one column and several keys) is, after packing to bf16, already the B-operand layout of
// the second product.  K rows are assigned to MFMA rows with bits 2 and 3 of the row index
// swapped; with that assignment the keys a lane holds are runs of eight consecutive tokens,
// matching one 16-byte piece of a dimension-major V row in the cache.
//
// K and V^T tiles are double-buffered in LDS: the global loads of tile i+1 are issued before the
// math of tile i and written to the other buffer afterwards (one barrier per tile).
//
// Scheduling.  Tiles of a sequence are processed in pairs (heaviest with lightest) by one
// workgroup so every workgroup of a causal prefill does the same amount of work; the long
// contexts of chunked prefill are additionally split into key ranges whose partial results are
// merged by launch_combine.
#include "internal.h"

#include <stdlib.h>

namespace shiftattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;
constexpr int kThreads = 256;
constexpr int kKvTile = kPrefillKvTile;           // 64 keys
constexpr int kKPitch = kD * 2 + 16;              // bytes per K row in LDS (padded)
constexpr int kVPitch = kKvTile * 2 + 16;         // bytes per V^T row in LDS (padded)
constexpr int kKBytes = kKvTile * kKPitch;        // 17408
constexpr int kVBytes = kD * kVPitch;             // 18432
constexpr int kStageBytes = kKBytes + kVBytes;    // 35840
constexpr int kLdsBytes = 2 * kStageBytes;        // 71680

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct PrefillParams {
    const uint16_t* q;
    const uint16_t* cache;
    const int32_t* block_table;
    const int32_t* cu_seqlens_q;
    const int32_t* seq_lens;
    uint16_t* out;
    float* o_part;
    float* ml_part;
    int64_t q_stride, out_stride;
    int num_seqs, total_q, hq_l, hkv_l, G;
    int gs_log2;      // log2 of heads stacked per token in the column index
    int head_slots;   // hq_l >> gs_log2
    int n_splits;     // key ranges per tile
    int max_blocks;
    float c;          // softmax_scale * log2(e)
};

template <int NQB>
__global__ __launch_bounds__(kThreads, NQB == 1 ? 2 : 1) void prefill_kernel(PrefillParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int kCols = 128 * NQB;  // columns per workgroup tile

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, half = lane >> 5;

    // ---- which (pair rank, key split, sequence, head slot) is this workgroup -----------------------
    const int n_sh = p.num_seqs * p.head_slots;
    int item = blockIdx.x;
    const int rank = item / (n_sh * p.n_splits);
    item -= rank * (n_sh * p.n_splits);
    const int split = item / n_sh;
    item -= split * n_sh;
    const int s = item / p.head_slots;
    const int hs = item - s * p.head_slots;

    const int q_begin = p.cu_seqlens_q[s];
    const int q_len = p.cu_seqlens_q[s + 1] - q_begin;
    const int ctx = p.seq_lens[s];
    const int tile_tokens = kCols >> p.gs_log2;
    const int n_tiles = (q_len + tile_tokens - 1) / tile_tokens;
    const int hi_tile = n_tiles - 1 - rank;
    if (rank > hi_tile) return;  // uniform
    const int n_pass = (hi_tile == rank) ? 1 : 2;
    const int gs_mask = (1 << p.gs_log2) - 1;
    const int g = (hs << p.gs_log2) / p.G;  // KV head of every column of this workgroup
    const int32_t* table = p.block_table + static_cast<size_t>(s) * p.max_blocks;
    const int last_block = (ctx - 1) / kBlockSize;

    // ---- global -> LDS mapping of this thread (one 16-byte piece of K and of V^T per cache block) --
    const int k_row = tid >> 4, k_piece = tid & 15;   // K block: 16 rows x 16 pieces
    const int v_row = tid >> 1, v_piece = tid & 1;    // V^T block: 128 rows x 2 pieces
    // ---- LDS -> MFMA operand mapping ------------------------------------------------------------------
    // K row feeding MFMA row l32: swap bits 2 and 3
    const int tau = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    const int k_rd = tau * kKPitch + half * 16;       // + sub*32*kKPitch + ks*32
    const int v_rd = l32 * kVPitch + half * 16;       // + mt*32*kVPitch + ks2*32

    int buf = 0;
    for (int pass = 0; pass < n_pass; ++pass) {
        const int tile = pass == 0 ? hi_tile : rank;
        const int tok0 = tile * tile_tokens;
        // ---- this lane's columns ------------------------------------------------------------------------
        int pos_col[NQB];     // position of the column's token in its sequence, -1 for padding columns
        int row_col[NQB];     // global row index (token) of the column
        int head_col[NQB];
        bf16x8 qf[NQB][8];
#pragma unroll
        for (int nb = 0; nb < NQB; ++nb) {
            const int cw = (wave * NQB + nb) * 32 + l32;
            const int tok = tok0 + (cw >> p.gs_log2);
            const bool valid = tok < q_len;
            head_col[nb] = (hs << p.gs_log2) + (cw & gs_mask);
            row_col[nb] = q_begin + tok;
            pos_col[nb] = valid ? ctx - q_len + tok : -1;
            const uint16_t* qp = p.q + static_cast<size_t>(row_col[nb]) * p.q_stride + head_col[nb] * kD + half * 8;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (valid) v = *reinterpret_cast<const u32x4*>(qp + ks * 16);
                qf[nb][ks] = as_bf16x8(v);
            }
        }
        // wavefront-uniform bounds of the wavefront's columns
        const int w_tok_first = tok0 + ((wave * NQB * 32) >> p.gs_log2);
        const int w_tok_last = min(tok0 + ((wave * NQB * 32 + NQB * 32 - 1) >> p.gs_log2), q_len - 1);
        const bool w_active = w_tok_first < q_len;
        const int w_pos_min = ctx - q_len + w_tok_first;
        const int w_pos_max = ctx - q_len + w_tok_last;

        // ---- key range of this (tile, split) ----------------------------------------------------------
        const int tile_pos_max = ctx - q_len + min(tok0 + tile_tokens, q_len) - 1;
        const int kv_tiles = tile_pos_max / kKvTile + 1;
        const int per_split = (kv_tiles + p.n_splits - 1) / p.n_splits;
        const int kt_begin = split * per_split;
        const int kt_end = min(kv_tiles, kt_begin + per_split);

        f32x16 oacc[NQB][4];
        float m_run[NQB], l_run[NQB];
#pragma unroll
        for (int nb = 0; nb < NQB; ++nb) {
            m_run[nb] = -INFINITY;
            l_run[nb] = 0.f;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[nb][mt][r] = 0.f;
        }

        u32x4 kreg[4], vreg[4];
        auto fetch = [&](int kt) {
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) {
                const int64_t blk = table[min(kt * 4 + bi, last_block)];
                kreg[bi] = *reinterpret_cast<const u32x4*>(p.cache + cache_part_offset(blk, g, 0, p.hkv_l, kD) + tid * 8);
                vreg[bi] = *reinterpret_cast<const u32x4*>(p.cache + cache_part_offset(blk, g, 1, p.hkv_l, kD) + tid * 8);
            }
        };
        auto stash = [&](int kt, unsigned char* stage) {
            const bool ragged = (kt + 1) * kKvTile > ctx;  // tile reaches past the context: uniform
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) {
                u32x4 v = vreg[bi];
                if (ragged) {
                    // keys at or past ctx were never written; clear their V so that 0 * x stays 0
                    const int n_valid = ctx - (kt * kKvTile + bi * 16 + v_piece * 8);
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        v[w] &= n_valid > 2 * w + 1 ? 0xFFFFFFFFu : (n_valid > 2 * w ? 0x0000FFFFu : 0u);
                }
                *reinterpret_cast<u32x4*>(stage + (bi * 16 + k_row) * kKPitch + k_piece * 16) = kreg[bi];
                *reinterpret_cast<u32x4*>(stage + kKBytes + v_row * kVPitch + bi * 32 + v_piece * 16) = v;
            }
        };

        if (kt_begin < kt_end) fetch(kt_begin);
        for (int kt = kt_begin; kt < kt_end; ++kt) {
            unsigned char* stage = lds + buf * kStageBytes;
            stash(kt, stage);
            __syncthreads();
            if (kt + 1 < kt_end) fetch(kt + 1);
            buf ^= 1;
            const int key0 = kt * kKvTile;
            if (!w_active || key0 > w_pos_max) continue;  // nothing visible for this wavefront (uniform)

            // ---- S^T = K Q^T ------------------------------------------------------------------------------
            f32x16 sacc[NQB][2];
#pragma unroll
            for (int nb = 0; nb < NQB; ++nb)
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sacc[nb][sub][r] = 0.f;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(stage + k_rd + sub * 32 * kKPitch + ks * 32));
#pragma unroll
                    for (int nb = 0; nb < NQB; ++nb)
                        sacc[nb][sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nb][ks], sacc[nb][sub], 0, 0, 0);
                }
            // accumulator register r of sub-tile sub holds key  key0 + 32*sub + 16*(r/8) + 8*half + r%8
            const bool need_mask = key0 + kKvTile - 1 > w_pos_min;
            bf16x8 pf[NQB][4];
#pragma unroll
            for (int nb = 0; nb < NQB; ++nb) {
                if (need_mask) {
#pragma unroll
                    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = key0 + 32 * sub + 16 * (r >> 3) + 8 * half + (r & 7);
                            if (key > pos_col[nb]) sacc[nb][sub][r] = -INFINITY;
                        }
                }
                float mx = -INFINITY;
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[nb][sub][r]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[nb], mx);
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;  // column with no visible key so far
                const float alpha = __builtin_amdgcn_exp2f((m_run[nb] - m_safe) * p.c);
                const float mc = m_safe * p.c;
                float psum = 0.f;
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float e = __builtin_amdgcn_exp2f(fmaf(sacc[nb][sub][r], p.c, -mc));
                        psum += e;
                        pf[nb][sub * 2 + (r >> 3)][r & 7] = static_cast<__bf16>(e);
                    }
                l_run[nb] = l_run[nb] * alpha + psum;
                m_run[nb] = m_new;
                if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {  // skip the rescale when no max moved
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[nb][mt][r] *= alpha;
                }
            }
            // ---- O^T += V^T P^T ---------------------------------------------------------------------------
#pragma unroll
            for (int ks2 = 0; ks2 < 4; ++ks2)
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) {
                    const bf16x8 a = as_bf16x8(
                        *reinterpret_cast<const u32x4*>(stage + kKBytes + v_rd + mt * 32 * kVPitch + ks2 * 32));
#pragma unroll
                    for (int nb = 0; nb < NQB; ++nb)
                        oacc[nb][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[nb][ks2], oacc[nb][mt], 0, 0, 0);
                }
        }

        // ---- epilogue: accumulator register r of row tile mt is head-dim  32*mt + 8*(r/4) + 4*half + r%4 ----
#pragma unroll
        for (int nb = 0; nb < NQB; ++nb) {
            const float l_tot = l_run[nb] + __shfl_xor(l_run[nb], 32);
            if (pos_col[nb] < 0) continue;
            if (p.n_splits == 1) {
                const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
                uint16_t* op = p.out + static_cast<size_t>(row_col[nb]) * p.out_stride + head_col[nb] * kD + 4 * half;
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                        bf16x4 v;
#pragma unroll
                        for (int x = 0; x < 4; ++x) v[x] = static_cast<__bf16>(oacc[nb][mt][r4 * 4 + x] * inv);
                        *reinterpret_cast<u32x2*>(op + 32 * mt + 8 * r4) = __builtin_bit_cast(u32x2, v);
                    }
            } else {
                const size_t prow = (static_cast<size_t>(split) * p.total_q + row_col[nb]) * p.hq_l + head_col[nb];
                float* op = p.o_part + prow * kD + 4 * half;
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        f32x4 v;
#pragma unroll
                        for (int x = 0; x < 4; ++x) v[x] = oacc[nb][mt][r4 * 4 + x];
                        *reinterpret_cast<f32x4*>(op + 32 * mt + 8 * r4) = v;
                    }
                if (half == 0) {
                    p.ml_part[prow * 2] = m_run[nb] * p.c;  // -inf when this key range held no visible key
                    p.ml_part[prow * 2 + 1] = l_tot;
                }
            }
        }
        __syncthreads();  // the next pass reuses both LDS buffers
    }
}

struct Plan {
    int nqb, gs_log2, head_slots, tile_tokens, pair_ranks, n_splits;
};

int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    return v ? atoi(v) : dflt;
}

Plan make_plan(int num_seqs, int total_q, int max_q_len, int max_seq_len, const AttnShape& a) {
    Plan pl;
    const int G = a.hq_l / a.hkv_l;
    const bool pow2 = (G & (G - 1)) == 0 && G <= 32;
    pl.gs_log2 = 0;
    if (pow2) while ((1 << pl.gs_log2) < G) ++pl.gs_log2;
    pl.head_slots = a.hq_l >> pl.gs_log2;
    pl.nqb = env_int("SHIFTATTN_PREFILL_NQB", 1) == 2 ? 2 : 1;
    pl.tile_tokens = (128 * pl.nqb) >> pl.gs_log2;
    const int tiles = (max_q_len + pl.tile_tokens - 1) / pl.tile_tokens;
    pl.pair_ranks = (tiles + 1) / 2;
    // Split the keys when the tiles alone cannot fill the chip (long cached context, short chunk).
    const long wgs = static_cast<long>((total_q + pl.tile_tokens - 1) / pl.tile_tokens + num_seqs) / 2 * pl.head_slots + 1;
    int splits = 1;
    const int forced = env_int("SHIFTATTN_PREFILL_SPLITS", 0);
    if (forced > 0) splits = forced;
    else if (wgs < 192) {
        const int by_fill = static_cast<int>((512 + wgs - 1) / wgs);
        const int by_len = max_seq_len / (8 * kKvTile);  // at least 8 key tiles per range
        splits = by_fill < by_len ? by_fill : by_len;
    }
    if (splits < 1) splits = 1;
    if (splits > 64) splits = 64;
    pl.n_splits = splits;
    return pl;
}

}  // namespace

bool prefill_mfma_supported(const AttnShape& a) { return a.elem == 2 && a.D == kD && a.hq_l % a.hkv_l == 0; }

size_t prefill_mfma_workspace(int num_seqs, int total_q, int max_q_len, int max_seq_len, const AttnShape& a) {
    const Plan pl = make_plan(num_seqs, total_q, max_q_len, max_seq_len, a);
    if (pl.n_splits == 1) return 0;
    return static_cast<size_t>(pl.n_splits) * total_q * a.hq_l * (kD + 2) * sizeof(float);
}

hipError_t launch_prefill_mfma(const void* q, const void* cache, const int32_t* block_table,
                               const int32_t* cu_seqlens_q, const int32_t* seq_lens, int num_seqs, int total_q,
                               int max_q_len, int max_seq_len, void* out, void* workspace, const AttnShape& a,
                               hipStream_t st) {
    if (num_seqs == 0 || total_q == 0 || max_q_len <= 0) return hipSuccess;
    const Plan pl = make_plan(num_seqs, total_q, max_q_len, max_seq_len, a);
    PrefillParams p;
    p.q = static_cast<const uint16_t*>(q);
    p.cache = static_cast<const uint16_t*>(cache);
    p.block_table = block_table;
    p.cu_seqlens_q = cu_seqlens_q;
    p.seq_lens = seq_lens;
    p.out = static_cast<uint16_t*>(out);
    const size_t part_rows = static_cast<size_t>(pl.n_splits) * total_q * a.hq_l;
    p.o_part = static_cast<float*>(workspace);
    p.ml_part = pl.n_splits > 1 ? p.o_part + part_rows * kD : nullptr;
    p.q_stride = a.q_stride;
    p.out_stride = a.out_stride;
    p.num_seqs = num_seqs;
    p.total_q = total_q;
    p.hq_l = a.hq_l;
    p.hkv_l = a.hkv_l;
    p.G = a.hq_l / a.hkv_l;
    p.gs_log2 = pl.gs_log2;
    p.head_slots = pl.head_slots;
    p.n_splits = pl.n_splits;
    p.max_blocks = a.max_blocks;
    p.c = a.scale * 1.4426950408889634f;

    const unsigned grid = static_cast<unsigned>(pl.pair_ranks) * pl.n_splits * num_seqs * pl.head_slots;
    hipError_t e;
    if (pl.nqb == 2) {
        static bool attr_done2 = false;
        if (!attr_done2) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel<2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
            if (e != hipSuccess) return e;
            attr_done2 = true;
        }
        prefill_kernel<2><<<grid, kThreads, kLdsBytes, st>>>(p);
    } else {
        static bool attr_done1 = false;
        if (!attr_done1) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel<1>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
            if (e != hipSuccess) return e;
            attr_done1 = true;
        }
        prefill_kernel<1><<<grid, kThreads, kLdsBytes, st>>>(p);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (pl.n_splits > 1)
        return launch_combine(p.o_part, p.ml_part, total_q, a.hq_l, kD, pl.n_splits, 0, nullptr, 0, out, a.out_stride,
                              a.elem, st);
    return hipSuccess;
}

}  // namespace shiftattn
