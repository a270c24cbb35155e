// Causal prefill attention of the local head shard over the paged KV cache (Algorithm 1, boxed
// attention line, prefill rows; chunked prefill continues a cached context).  bf16 tensors, fp32
// accumulation, head_dim 128.
//
// Tiling.  A workgroup owns a tile of 128 "columns"; a column is one (new token, query head) pair.
// The query heads that share a KV head are stacked next to each other in the column index (GS heads
// per token), so one K/V tile serves the whole GQA group and the causal diagonal of a tile spans
// only 128/GS tokens.  The workgroup has eight wavefronts in two groups of four: a wavefront owns 32
// columns, and the two groups split the key tiles (64 keys = four cache blocks each) of the column
// tile between them - group 0 takes the even tiles, group 1 the odd ones - and merge their
// partial results through LDS at the end.  That puts two wavefronts of the same workgroup on every
// SIMD (the matrix pipe and the vector ALUs only overlap across wavefronts: a lone wavefront hides
// about six vector instructions under one MFMA, measured) while the tile stays small enough that a
// 4 x 4096-token batch still yields one equal-work workgroup per compute unit.
//
// Math per key tile, transposed so that P never leaves registers:
//   S^T[key][col]  = K[key][:] . Q^T[:][col]     32x32x16 bf16 MFMA, A = K rows from LDS,
//                                                 B = Q^T held in registers for the whole tile
//   softmax down each column: a lane holds 32 keys of one column, the other 32 sit in lane+32, so
//   the column max costs one v_permlane32_swap
//   O^T[d][col]   += V^T[d][key] . P^T[key][col]  A = V^T rows from LDS, B = P^T straight from the
//                                                 softmax registers
// K rows are assigned to MFMA rows with bits 2 and 3 of the row index swapped; with that
// assignment the keys a lane holds are runs of eight consecutive tokens, matching one 16-byte piece
// of a dimension-major V row in the cache.
//
// Pipeline.  In iteration i a wavefront issues, interleaved in one instruction stream,
//   A(i+1): S^T of its next tile (16 MFMAs), B(i): softmax of the current tile (vector ALU),
//   C(i-1): O^T += V^T P^T of the previous tile (16 MFMAs),
// one MFMA, the LDS read of the operand two MFMAs ahead and a few softmax instructions at a time.
// Rescaling of O is lazy: a column's reference maximum only moves when the tile maximum exceeds it
// by more than 2^8 (in exp2 units), so `O *= alpha` is a rare wavefront-uniform branch; P then ranges
// up to 2^8, which bf16 and the fp32 sums hold without loss.
//
// Memory.  K and V^T tiles go from the cache to LDS with direct-to-LDS loads (no registers, no
// LDS store instructions), issued one iteration ahead of their use; a wavefront loads "its" cache
// block of the tile with eight 1-KiB loads that are contiguous in HBM.  LDS is not padded; bank
// conflicts are avoided by XOR-swizzling 16-byte pieces, applied on the global-address side of
// the load.  Stage `par` of a group is filled during an iteration of parity `par` and read during
// the next one; one barrier per iteration.
//
// Scheduling.  Tiles of a sequence are processed in pairs (heaviest with lightest) by one
// workgroup so every workgroup of a causal prefill does the same amount of work; the long
// contexts of chunked prefill are additionally split into key ranges whose partial results are
// merged by launch_combine.
#include "internal.h"

#include <utility>

namespace shiftattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;
constexpr int kThreads = 512;
constexpr int kKvTile = kPrefillKvTile;        // 64 keys
constexpr int kKBytes = kKvTile * kD * 2;      // 16384: K tile, 64 rows of 256 B
constexpr int kVBytes = kD * kKvTile * 2;      // 16384: V^T tile, 4 blocks of [128 rows][32 B]
constexpr int kStageBytes = kKBytes + kVBytes; // 32768
constexpr int kGroupBytes = 2 * kStageBytes;   // two stages per wavefront group
constexpr int kLdsBytes = 2 * kGroupBytes;     // 131072
constexpr int kBlockBytes = kBlockSize * kD * 2;  // 4096: K (or V^T) of one cache block and head

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

template <int kV>
struct IC {
    static constexpr int value = kV;
};

#define SHIFTATTN_INLINE __attribute__((always_inline))

// s_waitcnt vmcnt(0) with the other counters left alone (gfx9 encoding)
__device__ inline void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

struct PrefillParams {
    const uint16_t* __restrict__ q;
    const uint16_t* __restrict__ cache;
    const int32_t* __restrict__ block_table;
    const int32_t* __restrict__ cu_seqlens_q;
    const int32_t* __restrict__ seq_lens;
    uint16_t* __restrict__ out;
    float* __restrict__ o_part;
    float* __restrict__ ml_part;
    int64_t q_stride, out_stride;
    int num_seqs, total_q, hq_l, hkv_l, G;
    int gs_log2;      // log2 of heads stacked per token in the column index
    int head_slots;   // hq_l >> gs_log2
    int n_splits;     // key ranges per tile
    int rotate;       // the (sequence, head slot) index is rotated by the (pair rank, key range) index (see internal.h)
    int max_blocks;
    float c;          // softmax_scale * log2(e) (times k_scale for a cache widened from FP8)
    float out_scale;  // multiplies the normalised output: v_scale of an FP8 cache, else 1
};

__global__ __launch_bounds__(kThreads, 2) void prefill_kernel(PrefillParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int kCols = 128;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int grp = wave >> 2;  // key-tile parity this wavefront works on
    const int wg = wave & 3;    // column block of the wavefront; also the cache block of a tile it loads
    const int l32 = lane & 31, half = lane >> 5;

    // ---- which (pair rank, key split, sequence, head slot) is this workgroup -----------------------
    const int n_sh = p.num_seqs * p.head_slots;
    int item = blockIdx.x;
    const int rank = item / (n_sh * p.n_splits);
    item -= rank * (n_sh * p.n_splits);
    const int split = item / n_sh;
    item -= split * n_sh;
    if (p.rotate) item = (item + n_sh - static_cast<int>((blockIdx.x / n_sh) % n_sh)) % n_sh;
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
    const int32_t* __restrict__ table = p.block_table + static_cast<size_t>(s) * p.max_blocks;
    const int last_block = (ctx - 1) / kBlockSize;

    // ---- LDS addressing ---------------------------------------------------------------------------------
    unsigned char* gbase = lds + grp * kGroupBytes;  // this group's two stages
    // where this wavefront's direct-to-LDS loads land, as a scalar: the destination of such a load goes through M0,
    // and a per-lane copy of a wavefront-uniform value would cost vector ALU instructions at every load
    unsigned char* ld_base = lds + __builtin_amdgcn_readfirstlane(grp * kGroupBytes + wg * kBlockBytes);
    const int grp_u = __builtin_amdgcn_readfirstlane(grp), wg_u = __builtin_amdgcn_readfirstlane(wg);
    // K operand of MFMA row l32 is K row tau (bits 2 and 3 swapped); piece c of row r sits at c ^ (r & 15)
    const int tau = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    int k_rd[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) k_rd[ks] = tau * 256 + (((2 * ks + half) ^ (tau & 15)) << 4);
    // V^T operand: block-major [4][128 rows][32 B]; the two 16-byte halves of a row are swapped in
    // every other run of eight rows
    const int v_rd = kKBytes + l32 * 32 + ((half ^ ((l32 >> 3) & 1)) << 4);
    // direct-to-LDS loads: this wavefront fills cache block `wg` of a tile, 1 KiB per instruction
    // (LDS side contiguous in lane order; the swizzle is applied to the global address)
    int k_ld[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 4 * j + (lane >> 4);
        k_ld[j] = row * 256 + (((lane & 15) ^ row) << 4);
    }
    const int v_ld = kBlockBytes + (lane >> 1) * 32 + (((lane & 1) ^ ((lane >> 4) & 1)) << 4);
    const size_t blk_bytes = static_cast<size_t>(p.hkv_l) * 2 * kBlockBytes;
    // uniform values that the register allocator would otherwise keep in vector registers are pinned to scalar ones:
    // arithmetic on them then costs no vector instruction (each of which costs MFMA issue time in the key loop)
    auto uniform_ptr = [](const unsigned char* ptr) SHIFTATTN_INLINE -> const unsigned char* {
        const uint64_t a = reinterpret_cast<uint64_t>(ptr);
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
        return reinterpret_cast<const unsigned char*>((static_cast<uint64_t>(hi) << 32) | lo);
    };
    const unsigned char* cache_g =
        uniform_ptr(reinterpret_cast<const unsigned char*>(p.cache) + static_cast<size_t>(g) * 2 * kBlockBytes);

    typedef __attribute__((address_space(3))) void* lds_ptr;
    typedef const __attribute__((address_space(1))) void* glb_ptr;

    bf16x2 ones;
    ones[0] = static_cast<__bf16>(1.0f);
    ones[1] = static_cast<__bf16>(1.0f);
    const float thr = 8.0f / p.c;

    for (int pass = 0; pass < n_pass; ++pass) {
        const int tile = pass == 0 ? hi_tile : rank;
        const int tok0 = tile * tile_tokens;
        const int cw = wg * 32 + l32;
        const int tok = tok0 + (cw >> p.gs_log2);
        const bool valid = tok < q_len;
        const int head_col = (hs << p.gs_log2) + (cw & gs_mask);
        const int row_col = q_begin + tok;
        const int pos_col = valid ? ctx - q_len + tok : -1;
        bf16x8 qf[8];
        {
            const uint16_t* qp = p.q + static_cast<size_t>(row_col) * p.q_stride + head_col * kD + half * 8;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (valid) v = *reinterpret_cast<const u32x4*>(qp + ks * 16);
                qf[ks] = as_bf16x8(v);
            }
        }
        const int w_tok_first = tok0 + ((wg * 32) >> p.gs_log2);
        const int w_pos_min = __builtin_amdgcn_readfirstlane(w_tok_first < q_len ? ctx - q_len + w_tok_first : -1);

        // ---- key tiles of this (column tile, split), dealt alternately to the two groups ------------------
        const int tile_pos_max = ctx - q_len + min(tok0 + tile_tokens, q_len) - 1;
        const int kv_tiles = tile_pos_max / kKvTile + 1;
        const int per_split = (kv_tiles + p.n_splits - 1) / p.n_splits;
        const int kt_begin = split * per_split;
        const int kt_end = min(kv_tiles, kt_begin + per_split);
        const int n_all = max(kt_end - kt_begin, 0);
        const int n = (n_all + 1 - grp) >> 1;        // tiles of this group: kt(j) = kt_begin + grp + 2 j
        const int n_other = (n_all + grp) >> 1;
        // The tile that reaches past the context (if any) holds unwritten V slots; its owner clears them
        // in LDS before use, which costs one extra barrier that the other group mirrors.
        const bool pass_ragged = n_all > 0 && kt_end * kKvTile > ctx;
        const bool own_ragged = pass_ragged && (((n_all - 1) & 1) == grp);

        f32x16 oacc[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[mt][r] = 0.f;
        f32x16 sbuf[2][2];
        uint32_t pw[2][4][4];
        float m_used = -INFINITY, l_run = 0.f, alpha_pending = 1.f;

        auto kt_of = [&](int j) SHIFTATTN_INLINE { return kt_begin + grp_u + 2 * j; };
        // Cache block `wg` of the group's tile j.  Ids are fetched three tiles ahead and waited for a
        // whole iteration later: loads return in order, so a wait right behind the direct-to-LDS loads
        // (or right after the barrier) would stall for a full memory round trip every iteration.
        const int n_u = __builtin_amdgcn_readfirstlane(n);
        const int32_t* table_u = reinterpret_cast<const int32_t*>(uniform_ptr(reinterpret_cast<const unsigned char*>(table)));
        typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
        const const_i32_ptr table_c = (const_i32_ptr)table_u;
        auto fetch_id = [&](int j) SHIFTATTN_INLINE -> int {
            // every term of the address is uniform, and the table is read through the constant address space: the
            // compiler issues a scalar load, the id arrives in a scalar register without a vector instruction, and the
            // compiler itself places the wait in front of the first use (the bottom of the iteration, see below)
            const int idx = min((kt_begin + grp_u + 2 * min(j, max(n_u - 1, 0))) * 4 + wg_u, last_block);
            return table_c[idx];
        };
        auto id_arrived = [](int&) SHIFTATTN_INLINE {};   // the use itself waits
        auto block_base = [&](int id) SHIFTATTN_INLINE -> const unsigned char* {
            return cache_g + static_cast<int64_t>(id) * blk_bytes;
        };
        int id0 = 0, id1 = 0, id2 = 0;  // ids of tiles j, j+1, j+2 at the top of iteration j (uniform)
        // 1 KiB from src (wavefront-uniform, in scalar registers) + a 32-bit byte offset per lane + kImm into LDS at dst + kImm
        // (dst uniform): written as assembly so that the address is formed by the load itself (scalar base + vector offset)
        // instead of a 64-bit vector addition per load, which would cost MFMA issue time like any vector instruction.
        // The loads are waited for with explicit vmcnt(0) waits (wait_vm0) only.
        auto dma_1k = [&](const unsigned char* src, uint32_t lane_off, auto imm_c, unsigned char* dst) SHIFTATTN_INLINE {
            constexpr int kImm = decltype(imm_c)::value;
            const uint32_t m0v = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(dst));
            // (M0 is reserved by the compiler - it sets it right before each use of its own and keeps no value in it,
            // and rejects it on a clobber list - so writing it here needs no clobber.)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3"
                         :: "s"(m0v), "v"(lane_off), "s"(src), "n"(kImm) : "memory");
        };
        // the base must sit in scalar registers for the assembly above: said explicitly (it is wavefront-uniform, but the
        // register allocator may keep a uniform pointer in vector registers)
        auto scalar_ptr = [](const unsigned char* ptr) SHIFTATTN_INLINE -> const unsigned char* {
            const uint64_t a = reinterpret_cast<uint64_t>(ptr);
            const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
            const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
            return reinterpret_cast<const unsigned char*>((static_cast<uint64_t>(hi) << 32) | lo);
        };
        auto load_k = [&](const unsigned char* src_any, int stage) SHIFTATTN_INLINE {
            const unsigned char* src = scalar_ptr(src_any);
            unsigned char* dst = ld_base + stage * kStageBytes;
#pragma unroll
            for (int j = 0; j < 4; ++j) dma_1k(src, static_cast<uint32_t>(k_ld[j]), IC<0>{}, dst + j * 1024);
        };
        auto load_v = [&](const unsigned char* src_any, int stage) SHIFTATTN_INLINE {
            const unsigned char* src = scalar_ptr(src_any);
            unsigned char* dst = ld_base + stage * kStageBytes + kKBytes;
            // the instruction's immediate offset moves the LDS destination along with the source
            dma_1k(src, static_cast<uint32_t>(v_ld), IC<0>{}, dst);
            dma_1k(src, static_cast<uint32_t>(v_ld), IC<1024>{}, dst);
            dma_1k(src, static_cast<uint32_t>(v_ld), IC<2048>{}, dst);
            dma_1k(src, static_cast<uint32_t>(v_ld), IC<3072>{}, dst);
        };
        // zero the V^T entries of keys at or past the context in the given stage (tile kt)
        auto clear_ragged_v = [&](int kt, int stage) SHIFTATTN_INLINE {
            const int t4 = tid & 255;  // thread within the group
            const int d = t4 >> 1, h = t4 & 1;
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) {
                const int n_valid = ctx - (kt * kKvTile + bi * 16 + h * 8);
                if (n_valid < 8) {
                    u32x4* ptr = reinterpret_cast<u32x4*>(gbase + stage * kStageBytes + kKBytes + bi * kBlockBytes + d * 32 +
                                                          ((h ^ ((d >> 3) & 1)) << 4));
                    u32x4 v = *ptr;
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        v[w] &= n_valid > 2 * w + 1 ? 0xFFFFFFFFu : (n_valid > 2 * w ? 0x0000FFFFu : 0u);
                    *ptr = v;
                }
            }
        };
        auto apply_pending = [&]() SHIFTATTN_INLINE {
            if (__builtin_amdgcn_ballot_w64(alpha_pending != 1.f)) {
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[mt][r] *= alpha_pending;
            }
            alpha_pending = 1.f;
        };

        // One iteration on the group's tile j.  PAR = parity of j: selects register sets and LDS stages
        // at compile time (stage PAR is filled in this iteration, stage 1-PAR is read).
        auto body = [&](auto par_c, auto has_a_c, auto has_c_c, int j) SHIFTATTN_INLINE {
            constexpr int PAR = decltype(par_c)::value;
            constexpr bool HAS_A = decltype(has_a_c)::value != 0;
            constexpr bool HAS_C = decltype(has_c_c)::value != 0;
            constexpr int RD = 1 - PAR;
            f32x16(&s_cur)[2] = sbuf[PAR];
            f32x16(&s_nxt)[2] = sbuf[1 - PAR];
            uint32_t(&p_cur)[4][4] = pw[PAR];
            uint32_t(&p_prv)[4][4] = pw[1 - PAR];
            const int kt = kt_of(j);
            const int key0 = kt * kKvTile;

            constexpr int NOPS = (HAS_A ? 16 : 0) + (HAS_C ? 16 : 0);
            auto op_read = [&](auto tc) SHIFTATTN_INLINE -> u32x4 {
                constexpr int t = decltype(tc)::value;
                constexpr bool is_a = HAS_A && (!HAS_C || (t % 2 == 0));
                constexpr int o = (HAS_A && HAS_C) ? t / 2 : t;
                if constexpr (is_a)
                    return *reinterpret_cast<const u32x4*>(gbase + RD * kStageBytes + (o / 8) * 8192 + k_rd[o % 8]);
                else
                    return *reinterpret_cast<const u32x4*>(gbase + RD * kStageBytes + v_rd + (o / 4) * kBlockBytes + (o % 4) * 1024);
            };
            __syncthreads();
            // the operands of the first two MFMAs are requested first: their LDS latency passes while the loads below
            // are issued, instead of holding up the first MFMA behind the barrier
            u32x4 first0 = {0u, 0u, 0u, 0u}, first1 = first0;
            if constexpr (NOPS > 0) {
                first0 = op_read(IC<0>{});
                first1 = op_read(IC<1>{});
            }
            // fill stage PAR for the next iteration: K of tile j+2, V^T of tile j
            int id3_v = fetch_id(j + 3);  // consumed at the bottom of this iteration
            // In the steady state the two groups issue their loads at different times - the first group here, the second
            // behind its sixteenth MFMA: all eight wavefronts issuing at once queue up 64 KiB in the CU's one load path,
            // and a wavefront stuck at a load issues no MFMA; staggered, the other wavefront of its SIMD (which belongs to
            // the other group) keeps the pipe busy meanwhile.  Later than the middle of the step the loads would not
            // land before its end.
            constexpr bool kStagger = HAS_A && HAS_C;
            constexpr int kLateSlot = 16;
            const bool more_k = j + 2 < n;
            const unsigned char* k_src = block_base(id2);
            const unsigned char* v_src = block_base(id0);
            if (!kStagger || grp_u == 0) {
                if (more_k) load_k(k_src, PAR);
                load_v(v_src, PAR);
            }
            if (HAS_C) apply_pending();
            if (key0 + kKvTile - 1 > w_pos_min) {  // tile crosses the diagonal of this wavefront: uniform
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = key0 + 32 * sub + 16 * (r >> 3) + 8 * half + (r & 7);
                        if (key > pos_col) s_cur[sub][r] = -INFINITY;
                    }
            }

            // ---- interleaved block ------------------------------------------------------------------
            float mx = -INFINITY, mc = 0.f, alpha = 1.f, psum = 0.f;
            auto chunk = [&](auto cc) SHIFTATTN_INLINE {
                constexpr int c = decltype(cc)::value;
                if constexpr (c < 8) {
                    constexpr int sub = (4 * c) / 16, r = (4 * c) % 16;
                    mx = fmaxf(fmaxf(mx, s_cur[sub][r]), s_cur[sub][r + 1]);
                    mx = fmaxf(fmaxf(mx, s_cur[sub][r + 2]), s_cur[sub][r + 3]);
                } else if constexpr (c == 8) {
                    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                    // one v_max_f32: through fmaxf the two swapped halves would each be canonicalised first
                    asm("v_max_f32 %0, %1, %2" : "=v"(mx) : "v"(__uint_as_float(sw[0])), "v"(__uint_as_float(sw[1])));
                    const bool grow = mx > m_used + thr;
                    const float m_new = grow ? mx : m_used;
                    alpha = grow ? __builtin_amdgcn_exp2f((m_used - m_new) * p.c) : 1.f;
                    m_used = m_new;
                    mc = (m_new == -INFINITY ? 0.f : m_new) * p.c;
                    alpha_pending = alpha;
                    // the empty asm statements pin each result to its slot: without them the optimiser
                    // sinks the softmax below the MFMA sequence, next to its first use
                    asm volatile("" : "+v"(mc), "+v"(alpha), "+v"(m_used));
                } else if constexpr (c < 25) {
                    constexpr int v = 2 * (c - 9), sub = v / 16, r = v % 16;
                    const float e0 = __builtin_amdgcn_exp2f(fmaf(s_cur[sub][r], p.c, -mc));
                    const float e1 = __builtin_amdgcn_exp2f(fmaf(s_cur[sub][r + 1], p.c, -mc));
                    bf16x2 t;
                    t[0] = static_cast<__bf16>(e0);
                    t[1] = static_cast<__bf16>(e1);
                    psum = __builtin_amdgcn_fdot2_f32_bf16(t, ones, psum, false);
                    uint32_t w = __builtin_bit_cast(uint32_t, t);
                    asm volatile("" : "+v"(w), "+v"(psum));
                    p_cur[sub * 2 + (r >> 3)][(r & 7) >> 1] = w;
                } else {
                    l_run = l_run * alpha + psum;
                    asm volatile("" : "+v"(l_run));
                }
            };
            auto op_mfma = [&](auto tc, u32x4 a) SHIFTATTN_INLINE {
                constexpr int t = decltype(tc)::value;
                constexpr bool is_a = HAS_A && (!HAS_C || (t % 2 == 0));
                constexpr int o = (HAS_A && HAS_C) ? t / 2 : t;
                if constexpr (is_a) {
                    constexpr int sub = o / 8, ks = o % 8;
                    if constexpr (ks == 0) {
                        f32x16 z;
#pragma unroll
                        for (int r = 0; r < 16; ++r) z[r] = 0.f;
                        s_nxt[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), qf[ks], z, 0, 0, 0);
                    } else {
                        s_nxt[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), qf[ks], s_nxt[sub], 0, 0, 0);
                    }
                } else {
                    constexpr int ks2 = o / 4, mt = o % 4;
                    u32x4 pv = {p_prv[ks2][0], p_prv[ks2][1], p_prv[ks2][2], p_prv[ks2][3]};
                    oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(pv), oacc[mt], 0, 0, 0);
                }
            };

            if constexpr (NOPS == 0) {
                [&]<int... C>(std::integer_sequence<int, C...>) SHIFTATTN_INLINE { (chunk(IC<C>{}), ...); }
                (std::make_integer_sequence<int, 26>{});
            } else {
                u32x4 opnd[NOPS];
                opnd[0] = first0;
                opnd[1] = first1;
                [&]<int... T>(std::integer_sequence<int, T...>) SHIFTATTN_INLINE {
                    (([&]() SHIFTATTN_INLINE {
                         if constexpr (T + 2 < NOPS) opnd[T + 2] = op_read(IC<T + 2>{});
                         op_mfma(IC<T>{}, opnd[T]);
                         if constexpr (kStagger && T == kLateSlot) {
                             if (grp_u != 0) {
                                 if (more_k) load_k(k_src, PAR);
                                 load_v(v_src, PAR);
                             }
                         }
                         if constexpr (NOPS == 32) {
                             if constexpr (T < 26) chunk(IC<T>{});
                         } else {
                             if constexpr (2 * T < 26) chunk(IC<2 * T>{});
                             if constexpr (2 * T + 1 < 26) chunk(IC<2 * T + 1>{});
                         }
                         __builtin_amdgcn_sched_barrier(0);
                     }()),
                     ...);
                }
                (std::make_integer_sequence<int, NOPS>{});
            }
            wait_vm0();  // this wavefront's loads have landed before it reaches the next barrier
            id0 = id1;
            id1 = id2;
            id_arrived(id3_v);
            id2 = id3_v;
        };

        int barriers = 0;  // barriers this group executes in the pass; both groups must end up equal
        if (n > 0) {
            // prologue: K of the first two tiles, S^T of the first
            {
                int a0 = fetch_id(0), a1 = fetch_id(1), a2 = fetch_id(2);
                id_arrived(a0);
                id_arrived(a1);
                id_arrived(a2);
                id0 = a0;
                id1 = a1;
                id2 = a2;
                load_k(block_base(id0), 0);
                if (n > 1) load_k(block_base(id1), 1);
            }
            wait_vm0();
            __syncthreads();
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sbuf[0][sub][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const u32x4 a = *reinterpret_cast<const u32x4*>(gbase + sub * 8192 + k_rd[ks]);
                    sbuf[0][sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), qf[ks], sbuf[0][sub], 0, 0, 0);
                }
            }
            if (n == 1) {
                body(IC<0>{}, IC<0>{}, IC<0>{}, 0);
            } else {
                body(IC<0>{}, IC<1>{}, IC<0>{}, 0);
                int j = 1;  // stays odd: the steady-state loop takes two tiles per trip so that the
                            // register sets of even and odd tiles are fixed at compile time
                for (; j + 2 < n; j += 2) {
                    body(IC<1>{}, IC<1>{}, IC<1>{}, j);
                    body(IC<0>{}, IC<1>{}, IC<1>{}, j + 1);
                }
                if (j + 1 < n) {
                    body(IC<1>{}, IC<1>{}, IC<1>{}, j);
                    body(IC<0>{}, IC<0>{}, IC<1>{}, j + 1);
                } else {
                    body(IC<1>{}, IC<0>{}, IC<1>{}, j);
                }
            }
            // epilogue: C of the last tile
            __syncthreads();
            const int lp = (n - 1) & 1;
            if (own_ragged) {
                clear_ragged_v(kt_of(n - 1), lp);
                __syncthreads();
            }
            apply_pending();
            auto last_c = [&](auto par_c) SHIFTATTN_INLINE {
                constexpr int PAR = decltype(par_c)::value;
#pragma unroll
                for (int ks2 = 0; ks2 < 4; ++ks2)
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt) {
                        const u32x4 a = *reinterpret_cast<const u32x4*>(gbase + PAR * kStageBytes + v_rd + ks2 * kBlockBytes + mt * 1024);
                        u32x4 pv = {pw[PAR][ks2][0], pw[PAR][ks2][1], pw[PAR][ks2][2], pw[PAR][ks2][3]};
                        oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(pv), oacc[mt], 0, 0, 0);
                    }
            };
            if (lp) last_c(IC<1>{});
            else last_c(IC<0>{});
            barriers = n + 2 + (own_ragged ? 1 : 0);
        }
        // even out the barrier count of the two groups (their LDS regions are disjoint, only the count matters)
        const int other_barriers = n_other > 0 ? n_other + 2 + ((pass_ragged && !own_ragged) ? 1 : 0) : 0;
        for (int b = barriers; b < other_barriers; ++b) __syncthreads();

        // ---- merge the two groups -------------------------------------------------------------------------
        float l_tot = l_run + __shfl_xor(l_run, 32);
        __syncthreads();  // every wavefront is done with the tile stages
        // the thread index is read through an opaque copy: addresses derived from the plain value are loop
        // invariants that the optimiser computes before the key loop and then spills around it
        int tid_m = tid;
        asm volatile("" : "+v"(tid_m));
        const int t4 = tid_m & 255;
        if (p.n_splits == 1) {
            // Each group finishes one half of the head dimension (group 0 rows 0..63, group 1 rows 64..127): it parks
            // the other half of its accumulators for the other group, folds in what that group parked, normalises,
            // and puts bf16 rows into an LDS staging tile; then all eight wavefronts write the tile out in whole
            // 256-byte rows (one 16-byte piece per lane, 1 KiB of consecutive output per instruction per 4 rows).
            float* park = reinterpret_cast<float*>(lds);                 // [2 groups][32 values][256 lanes]
            float* x_ml = park + 2 * 32 * 256;                            // [2 groups][2][256]
            constexpr int kPitch = 272;                                   // staging row pitch in bytes (256 + 16)
            unsigned char* stage = lds + (2 * 32 * 256 + 2 * 2 * 256) * 4;  // [128 columns][kPitch]
            // (register arrays are indexed with compile-time constants only: one copy of the code per group)
            auto park_half = [&](auto g_c) SHIFTATTN_INLINE {
                constexpr int GRP = decltype(g_c)::value;
                float* mine = park + GRP * (32 * 256);
#pragma unroll
                for (int k = 0; k < 2; ++k)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mine[(k * 16 + r) * 256 + t4] = oacc[2 * (1 - GRP) + k][r];
                x_ml[(GRP * 2) * 256 + t4] = m_used;
                x_ml[(GRP * 2 + 1) * 256 + t4] = l_tot;
            };
            if (grp == 0) park_half(IC<0>{});
            else park_half(IC<1>{});
            __syncthreads();
            auto finish_half = [&](auto g_c) SHIFTATTN_INLINE {
                constexpr int grp = decltype(g_c)::value;  // shadows the runtime value
                const float* theirs = park + (1 - grp) * (32 * 256);
                const float m_o = x_ml[((1 - grp) * 2) * 256 + t4], l_o = x_ml[((1 - grp) * 2 + 1) * 256 + t4];
                const float m_star = fmaxf(m_used, m_o);
                const float w_me = m_used == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m_used - m_star) * p.c);
                const float w_o = m_o == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m_o - m_star) * p.c);
                const float l_all = l_tot * w_me + l_o * w_o;
                const float inv = l_all > 0.f ? p.out_scale / l_all : 0.f;
                const float a_me = w_me * inv, a_o = w_o * inv;
                const int cw_m = ((tid_m >> 6) & 3) * 32 + (tid_m & 31), half_m = (tid_m >> 5) & 1;
                unsigned char* srow = stage + cw_m * kPitch + (64 * grp + 4 * half_m) * 2;
#pragma unroll
                for (int k = 0; k < 2; ++k)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        bf16x4 v;
#pragma unroll
                        for (int x = 0; x < 4; ++x)
                            v[x] = static_cast<__bf16>(oacc[2 * grp + k][r4 * 4 + x] * a_me + theirs[(k * 16 + r4 * 4 + x) * 256 + t4] * a_o);
                        *reinterpret_cast<u32x2*>(srow + (32 * k + 8 * r4) * 2) = __builtin_bit_cast(u32x2, v);
                    }
            };
            if (grp == 0) finish_half(IC<0>{});
            else finish_half(IC<1>{});
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int col = (tid_m >> 4) + 32 * i, piece = tid_m & 15;
                const int tok_c = tok0 + (col >> p.gs_log2);
                if (tok_c < q_len) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(stage + col * kPitch + piece * 16);
                    uint16_t* op = p.out + static_cast<size_t>(q_begin + tok_c) * p.out_stride +
                                   ((hs << p.gs_log2) + (col & gs_mask)) * kD + piece * 8;
                    *reinterpret_cast<u32x4*>(op) = v;
                }
            }
        } else {
            // key ranges split over workgroups: group 1 parks (m, l, O) in LDS, group 0 folds it in and writes the
            // un-normalised partial of this range
            float* x_o = reinterpret_cast<float*>(lds);                   // [64 values][256 lanes of a group]
            float* x_ml = x_o + 64 * 256;                                  // [2][256]
            if (grp == 1) {
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) x_o[(mt * 16 + r) * 256 + t4] = oacc[mt][r];
                x_ml[t4] = m_used;
                x_ml[256 + t4] = l_tot;
            }
            __syncthreads();
            if (grp == 0) {
                const float m1 = x_ml[t4], l1 = x_ml[256 + t4];
                const float m_star = fmaxf(m_used, m1);
                const float w0 = m_used == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m_used - m_star) * p.c);
                const float w1 = m1 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m1 - m_star) * p.c);
                l_tot = l_tot * w0 + l1 * w1;
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[mt][r] = oacc[mt][r] * w0 + x_o[(mt * 16 + r) * 256 + t4] * w1;
                if (pos_col >= 0) {
                    // accumulator register r of row tile mt is head-dim 32*mt + 8*(r/4) + 4*half + r%4
                    const size_t prow = (static_cast<size_t>(split) * p.total_q + row_col) * p.hq_l + head_col;
                    float* op = p.o_part + prow * kD + 4 * half;
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            f32x4 v;
#pragma unroll
                            for (int x = 0; x < 4; ++x) v[x] = oacc[mt][r4 * 4 + x];
                            *reinterpret_cast<f32x4*>(op + 32 * mt + 8 * r4) = v;
                        }
                    if (half == 0) {
                        p.ml_part[prow * 2] = m_star * p.c;  // -inf when this key range held no visible key
                        p.ml_part[prow * 2 + 1] = l_tot;
                    }
                }
            }
        }
        __syncthreads();  // the next pass reuses LDS
    }
}

constexpr double kPassSeconds = 7e-6;  // what a pass of this kernel costs around its key loop (Q, first tiles, merge of the groups, write-out)

struct Plan {
    int gs_log2, head_slots, tile_tokens, pair_ranks, n_splits;
    bool rotate;
};

Plan make_plan(int num_seqs, int total_q, int max_q_len, int max_seq_len, const AttnShape& a) {
    Plan pl;
    const int G = a.hq_l / a.hkv_l;
    const bool pow2 = (G & (G - 1)) == 0 && G <= 32;
    pl.gs_log2 = 0;
    if (pow2) while ((1 << pl.gs_log2) < G) ++pl.gs_log2;
    pl.head_slots = a.hq_l >> pl.gs_log2;
    pl.tile_tokens = 128 >> pl.gs_log2;
    const int tiles = (max_q_len + pl.tile_tokens - 1) / pl.tile_tokens;
    pl.pair_ranks = (tiles + 1) / 2;
    // Key ranges per column tile: the count that minimises the model of a launch that also decides between the two
    // kernels - more ranges when the tiles alone cannot fill the chip (long cached context, short chunk) or fill it
    // with a ragged last round (320 equal workgroups on 256 compute units), as long as the merge does not eat the gain.
    const long wgs = static_cast<long>(pl.pair_ranks) * num_seqs * pl.head_slots;
    int splits = 1;
    const int forced = option_prefill_splits();
    if (forced > 0) {
        splits = forced;
    } else {
        const int by_len = max_seq_len / (16 * kKvTile);  // at least 16 key tiles per range
        const double walks = paired_walks(max_q_len, max_seq_len);
        // (with what the passes cost around their key loops: two per round of pairs, about 7 us each)
        auto priced = [&](int sp) {
            return launch_model_seconds(wgs, sp, 128, total_q, max_seq_len, a.hq_l, walks) +
                   2.0 * static_cast<double>((wgs * sp + 255) / 256) * kPassSeconds;
        };
        double best = priced(1);
        for (int cand = 2; cand <= 16 && cand <= by_len; ++cand) {
            const double t = priced(cand);
            if (t < best * 0.97) {  // a further range must pay for itself
                best = t;
                splits = cand;
            }
        }
    }
    if (splits < 1) splits = 1;
    if (splits > 64) splits = 64;
    pl.n_splits = splits;
    pl.rotate = rotate_sequences_over_dies(num_seqs, pl.head_slots, total_q, max_q_len);
    return pl;
}

// FP8 E4M3 cache: the blocks the batch reads are first widened to bf16 (exact) into a scratch cache in
// the workspace, block i of sequence s at scratch block s * nb + i with nb = blocks of the longest
// context, together with the block table that says so; the kernel then runs on the scratch cache with
// k_scale in its logit scale and v_scale on its output.  The pass moves 1.5 bytes per cached element
// once, against the 4 * D flops per (query, key) pair of the attention itself.
constexpr size_t kFp8ScratchLimit = static_cast<size_t>(8) << 30;  // larger batches take the general kernel

struct Fp8Scratch {
    int nb;               // scratch blocks per sequence
    size_t cache_bytes;   // bf16 scratch cache
    size_t table_bytes;   // int32 [num_seqs][nb], padded to 256 bytes
};

Fp8Scratch fp8_scratch(int num_seqs, int max_seq_len, const AttnShape& a) {
    Fp8Scratch f;
    f.nb = (max_seq_len + kBlockSize - 1) / kBlockSize;
    f.cache_bytes = static_cast<size_t>(num_seqs) * f.nb * a.hkv_l * 2 * kBlockBytes;
    f.table_bytes = (static_cast<size_t>(num_seqs) * f.nb * sizeof(int32_t) + 255) / 256 * 256;
    return f;
}

}  // namespace

bool prefill_mfma_supported(const AttnShape& a, int num_seqs, int max_seq_len) {
    if (!(a.elem == 2 && a.D == kD && a.hq_l % a.hkv_l == 0)) return false;
    return !a.kv_fp8() || fp8_scratch(num_seqs, max_seq_len, a).cache_bytes <= kFp8ScratchLimit;
}

namespace {

// Which of the two kernels serves a launch.  The 256-column kernel is the faster one per MFMA (about 12 %), but its tiles
// are twice as large: a batch like 4 x 4096 tokens with 4 query heads per KV head makes 128 pairs of 256-column tiles and
// 256 pairs of 128-column tiles, and only the latter cover the chip with equal workgroups and no merge pass.  The choice
// compares the two plans under the same rough model of a launch.
struct Choice {
    bool wide;
    Plan narrow;
    Prefill64Plan w;
};

Choice choose(int num_seqs, int total_q, int max_q_len, int max_seq_len, const AttnShape& a) {
    Choice c;
    c.narrow = make_plan(num_seqs, total_q, max_q_len, max_seq_len, a);
    c.wide = false;
    // (a cache widened from FP8 is bf16 by the time a kernel runs, so only the other conditions matter)
    AttnShape b = a;
    b.kv_elem = b.elem;
    if (!prefill_mfma64_supported(b)) return c;
    c.w = prefill_mfma64_plan(num_seqs, total_q, max_q_len, max_seq_len, a, option_prefill_splits());
    const int forced = option_prefill_tile();
    if (forced == 128) return c;
    // Both priced with what their passes cost around the key loop (two passes per round of pairs here; the wide kernel's,
    // about 15 us each, are in its plan); the 12 % are this kernel's slower loop.  The workgroups that weigh are counted
    // as for the wide kernel: those of sequences shorter than the longest are light or leave at once.
    const long wgs_n = static_cast<long>(c.narrow.pair_ranks * longest_chunk_equivalents(num_seqs, total_q, max_q_len) * c.narrow.head_slots + 0.999);
    const double rounds_n = static_cast<double>((wgs_n * c.narrow.n_splits + 255) / 256);
    const double t_narrow = 1.12 * launch_model_seconds(wgs_n, c.narrow.n_splits, 128, total_q, max_seq_len, a.hq_l,
                                                         paired_walks(max_q_len, max_seq_len)) + 2.0 * rounds_n * kPassSeconds;
    c.wide = forced == 256 || c.w.model_with_passes < 0.97 * t_narrow;
    return c;
}

size_t split_bytes_of(const Choice& c, int total_q, const AttnShape& a) {
    if (c.wide) return prefill_mfma64_workspace(total_q, c.w, a);
    return c.narrow.n_splits == 1 ? 0 : static_cast<size_t>(c.narrow.n_splits) * total_q * a.hq_l * (kD + 2) * sizeof(float);
}

}  // namespace

size_t prefill_mfma_workspace(int num_seqs, int total_q, int max_q_len, int max_seq_len, const AttnShape& a) {
    const Choice c = choose(num_seqs, total_q, max_q_len, max_seq_len, a);
    size_t bytes = split_bytes_of(c, total_q, a);
    if (a.kv_fp8()) {
        const Fp8Scratch f = fp8_scratch(num_seqs, max_seq_len, a);
        bytes = (bytes + 255) / 256 * 256 + f.cache_bytes + f.table_bytes;
    }
    return bytes;
}

hipError_t prefill_mfma_init() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               kLdsBytes);
}

hipError_t launch_prefill_mfma(const void* q, const void* cache, const int32_t* block_table,
                               const int32_t* cu_seqlens_q, const int32_t* seq_lens, int num_seqs, int total_q,
                               int max_q_len, int max_seq_len, void* out, void* workspace, const AttnShape& a,
                               hipStream_t st) {
    if (num_seqs == 0 || total_q == 0 || max_q_len <= 0) return hipSuccess;
    const Choice ch = choose(num_seqs, total_q, max_q_len, max_seq_len, a);
    int max_blocks = a.max_blocks;
    if (a.kv_fp8()) {  // widen into the scratch cache behind the split partials, then attend over that
        const Fp8Scratch f = fp8_scratch(num_seqs, max_seq_len, a);
        const size_t split_bytes = (split_bytes_of(ch, total_q, a) + 255) / 256 * 256;
        unsigned char* scratch = static_cast<unsigned char*>(workspace) + split_bytes;
        int32_t* table2 = reinterpret_cast<int32_t*>(scratch + f.cache_bytes);
        hipError_t e0 = launch_fp8_blocks_to_bf16(cache, block_table, a.max_blocks, seq_lens, num_seqs, f.nb, a.hkv_l, scratch,
                                                 table2, st);
        if (e0 != hipSuccess) return e0;
        cache = scratch;
        block_table = table2;
        max_blocks = f.nb;
    }
    const float c = a.scale * a.k_scale * 1.4426950408889634f;
    if (ch.wide)
        return launch_prefill_mfma64(q, cache, block_table, max_blocks, cu_seqlens_q, seq_lens, num_seqs, total_q, ch.w, out,
                                     workspace, a, c, a.v_scale, st);
    const Plan& pl = ch.narrow;
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
    p.rotate = pl.rotate ? 1 : 0;
    p.max_blocks = max_blocks;
    p.c = c;
    p.out_scale = a.v_scale;

    const unsigned grid = static_cast<unsigned>(pl.pair_ranks) * pl.n_splits * num_seqs * pl.head_slots;
    prefill_kernel<<<grid, kThreads, kLdsBytes, st>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (pl.n_splits > 1)
        return launch_combine(p.o_part, p.ml_part, total_q, a.hq_l, kD, pl.n_splits, 0, nullptr, 0, out, a.out_stride,
                              a.elem, a.v_scale, st);
    return hipSuccess;
}

}  // namespace shiftattn
