// Causal prefill attention of the local head shard over the paged KV cache (Algorithm 1, boxed attention line,
// prefill rows; chunked prefill continues a cached context): the wide-tile kernel.  bf16 tensors, fp32
// accumulation, head_dim 128, bf16 cache.
//
// One wavefront per SIMD, 64 columns per wavefront.  A workgroup is four wavefronts and owns a tile of 256
// "columns"; a column is one (new token, query head) pair, the G query heads that share a KV head lying next to
// each other (column = token * G + head, any G up to 256), so one K/V tile serves the whole GQA group.  All four
// wavefronts walk the same keys, 32 at a time (two cache blocks), and share every K and V^T tile through LDS:
// against a 128-column tile with 32-column wavefronts this halves the bytes that go from the cache into LDS per
// MFMA, halves the operand bytes read from LDS per MFMA (an operand read feeds two MFMAs, one per 32-column
// block) and halves the barriers per SIMD.  The price is registers - Q^T (64), O^T (128), two S^T tiles (64) and
// two P^T tiles (32) per lane - which is why only one wavefront fits a SIMD; the matrix pipe and the vector ALU
// then overlap inside the one instruction stream, which is written out slot by slot (one MFMA, the softmax work
// of one logit, a share of the operand reads).
//
// Math per key tile, transposed so that P never leaves registers (as in the 128-column kernel):
//   S^T[key][col]  = K[key][:] . Q^T[:][col]      32x32x16 bf16 MFMA, A = K rows from LDS, B = Q^T in registers
//   O^T[d][col]   += V^T[d][key] . P^T[key][col]  A = V^T rows from LDS, B = P^T straight from the softmax
// with bits 2 and 3 of the K row index swapped in the MFMA row assignment, so that the keys a lane holds are runs
// of eight consecutive tokens (one 16-byte piece of a dimension-major V row).
//
// Softmax against a reference that lags.  Softmax does not care which reference its exponentials are shifted by as long
// as nothing leaves the range of bf16 and the fp32 sums.  The first attempt at a pass takes the reference from the
// column's first visible key tile (whose maximum then gets P = 1 exactly: a row with few keys, all in that tile, comes
// out as exactly as the careful way would give it) and follows no maximum behind it: a fused multiply-add, an
// exponential and the row sum per logit, one packing per two, is all the loop spends on the softmax.  Real logits stay
// within 2^100 of their first tile's maximum, and P up to 2^100 is held by bf16 and the fp32 sums without loss; a column
// whose sum ends beyond that flags the pass, which is then run again the careful way: the exponentials of a tile are
// taken against the column's reference maximum as it stood when the tile began (so they do not wait for the tile's own
// maximum and spread evenly over the MFMA slots), the tile's maximum is collected on the side and checked against the
// reference (slack 2^32): a column that has no sums yet takes a new reference and recomputes the tile's P from the S^T
// values it still holds, one that has sums flags the pass once more, and the third attempt starts from references
// within the slack of every column's true maximum.  O^T is never rescaled inside the loop.
// A process-wide switch (off by default) makes the first attempt cheaper still: Q^T is multiplied by the softmax scale
// when the tile fetches it and rounded to bf16 again, the logits leave the MFMAs in exp2 units, and P is the exp2 of
// the logit itself, with no reference at all (sums must end inside [2^-40, 2^40]).  A logit then moves by up to 2^-9 of
// its value and the largest P is no longer exactly 1, which can put an output of magnitude 2 or more one bf16 step from
// the correctly rounded value; a pass that is flagged fetches Q^T again as given.
//
// Pipeline of iteration j: S^T of tile j+1 (16 MFMAs), softmax of tile j, O^T += V^T P^T of tile j-1 (16 MFMAs).
// LDS holds a ring of three stages of K (32 keys) + V^T (32 keys), tile t in stage t%3.  During iteration j
// wavefronts 0 and 1 bring K of tile j+3 (one cache block each) and wavefronts 2 and 3 V^T of tile j+1, by
// direct-to-LDS loads; what iteration j reads was loaded two iterations earlier and made visible by the barrier of
// the iteration before, so operand reads and MFMAs run on across the one barrier per iteration (which sits a few
// slots into the iteration, in front of the loads that overwrite the stage everybody has just left).  With a single
// wavefront per SIMD every instruction of the iteration - barrier, loads, address updates, the check of the maximum -
// takes issue time the MFMAs cannot hide behind another wavefront, so all of it is kept to a few instructions.
//
// Scheduling: tiles of a sequence are processed in pairs (heaviest with lightest) by one workgroup; a short chunk on a
// long context is taken one tile per workgroup, its keys split into ranges merged by launch_combine.
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
constexpr int kThreads = 256;
constexpr int kCols = 256;                     // columns of a workgroup tile
constexpr int kKv = 32;                        // keys per iteration
constexpr int kKBytes = kKv * kD * 2;          // 8192: K tile, 32 rows of 256 B
constexpr int kVBytes = kD * kKv * 2;          // 8192: V^T tile, 2 blocks of [128 rows][32 B]
constexpr int kStageBytes = kKBytes + kVBytes; // 16384
constexpr int kRingBytes = 3 * kStageBytes;    // 49152
constexpr int kBlockBytes = kBlockSize * kD * 2;  // 4096: K (or V^T) of one cache block and head
constexpr int kPitch = 272;                    // row pitch of the output staging tile (256 + 16 bytes)
constexpr int kFlagBytes = 16;                 // one redo flag per wavefront
constexpr int kLdsBytes = kRingBytes + kCols * kPitch + kFlagBytes;  // 118800
// A column's reference maximum may lag its true running maximum by this much (exp2 units): P reaches 2^32 at most, far
// inside what bf16 and the fp32 sums hold (their relative precision does not depend on magnitude); O^T overflows only
// for |V| beyond 2^70.
constexpr float kRefSlack = 32.0f;
// The first attempt at a pass uses no reference (see the top of the file): the sum of a column that sees keys must end
// inside this range - its largest P then lies within a factor "number of keys" of the sum, far from bf16's denormals and
// from overflow (O^T overflows only for |V| beyond 2^87), and every logit that matters lies within 40 + log2(keys) of
// zero (which also bounds what a second rounding of Q^T can move).  An infinity or a NaN fails the test.
constexpr float kFreeSumLo = 0x1p-40f, kFreeSumHi = 0x1p40f;
// The default first attempt keeps the reference the column's first key tile left and follows no maximum behind it: P may
// then reach 2^100 (still far inside bf16 and fp32 range; O^T overflows only for |V| beyond 2^27), and a sum beyond that
// sends the pass to the attempts that do follow the maximum.
constexpr float kKeepSumBound = 0x1p100f;

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

template <int kV>
struct IC {
    static constexpr int value = kV;
};

#define SHIFTATTN_INLINE __attribute__((always_inline))
#define SHIFTATTN_FORCE_INLINE inline __attribute__((always_inline))

// s_waitcnt vmcnt(0) with the other counters left alone (gfx9 encoding)
__device__ inline void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// The matrix instructions are written as assembly to fix where their accumulators live: S^T in ordinary vector
// registers (the softmax reads every element with the vector ALU), O^T in accumulation registers (touched by
// nothing but MFMAs in the steady state), Q^T (a B operand) in accumulation registers as well.  Left to itself the
// compiler gives all MFMA results of a function to one register file and copies S^T across, one extra vector
// instruction per logit.  The compiler does not see that these statements are MFMAs, so it inserts none of the wait
// states a reader of their result needs (11 for an 8-pass MFMA): every place where compiler-generated code reads
// such a result sits behind at least that many instructions, and mfma_settle() is put where that is not evident.
// The same blindness works the other way: where the compiler itself writes an MFMA source right in front of such a
// statement (it moves accumulators between registers where differently allocated copies of the loop body meet) it adds
// no wait state either, and the MFMA reads a stale register.  kGuard puts the wait states into the statement; every
// MFMA outside the steady-state loop is guarded, the loop itself has no such writes (its accumulators never move).
template <bool kGuard>
__device__ SHIFTATTN_FORCE_INLINE void mfma_s_first(f32x16& d, u32x4 a, bf16x8 b) {
    if constexpr (kGuard) asm volatile("s_nop 4\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
}
template <bool kGuard>
__device__ SHIFTATTN_FORCE_INLINE void mfma_s_acc(f32x16& d, u32x4 a, bf16x8 b) {
    if constexpr (kGuard) asm volatile("s_nop 4\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
}
template <bool kGuard>
__device__ SHIFTATTN_FORCE_INLINE void mfma_o_acc(f32x16& d, u32x4 a, u32x4 b) {
    if constexpr (kGuard) asm volatile("s_nop 4\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}
__device__ SHIFTATTN_FORCE_INLINE void mfma_settle() { asm volatile("s_nop 7\n\ts_nop 7" ::: "memory"); }

// Q^T of a lane - eight 16-byte pieces for each of its two column blocks, 32 bytes apart - from global memory straight
// into accumulation registers, where the MFMAs take it as their B operand (a value that is born in ordinary registers
// and only used from accumulation registers is copied across at every use).  One statement with its own wait: the
// compiler does not know these are loads, so the registers must hold their values when the statement ends.
__device__ SHIFTATTN_FORCE_INLINE void load_q_to_acc(bf16x8 (&q0)[8], bf16x8 (&q1)[8], const void* p0, const void* p1) {
    asm volatile(
        "global_load_dwordx4 %0, %16, off\n\tglobal_load_dwordx4 %1, %16, off offset:32\n\t"
        "global_load_dwordx4 %2, %16, off offset:64\n\tglobal_load_dwordx4 %3, %16, off offset:96\n\t"
        "global_load_dwordx4 %4, %16, off offset:128\n\tglobal_load_dwordx4 %5, %16, off offset:160\n\t"
        "global_load_dwordx4 %6, %16, off offset:192\n\tglobal_load_dwordx4 %7, %16, off offset:224\n\t"
        "global_load_dwordx4 %8, %17, off\n\tglobal_load_dwordx4 %9, %17, off offset:32\n\t"
        "global_load_dwordx4 %10, %17, off offset:64\n\tglobal_load_dwordx4 %11, %17, off offset:96\n\t"
        "global_load_dwordx4 %12, %17, off offset:128\n\tglobal_load_dwordx4 %13, %17, off offset:160\n\t"
        "global_load_dwordx4 %14, %17, off offset:192\n\tglobal_load_dwordx4 %15, %17, off offset:224\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&a"(q0[0]), "=&a"(q0[1]), "=&a"(q0[2]), "=&a"(q0[3]), "=&a"(q0[4]), "=&a"(q0[5]), "=&a"(q0[6]), "=&a"(q0[7]),
          "=&a"(q1[0]), "=&a"(q1[1]), "=&a"(q1[2]), "=&a"(q1[3]), "=&a"(q1[4]), "=&a"(q1[5]), "=&a"(q1[6]), "=&a"(q1[7])
        : "v"(p0), "v"(p1)
        : "memory");
}

// block tables are read through the constant address space: with a wavefront-uniform index the compiler then issues
// scalar loads (and places the waits itself)
typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
// operand reads take their LDS address as a plain 32-bit number (formed once from the array's base): indexing the
// shared array with a register costs a vector addition of the base per read
typedef const __attribute__((address_space(3))) u32x4* lds_u32x4_ptr;
__device__ SHIFTATTN_FORCE_INLINE u32x4 lds_read16(int addr) {
    return *(lds_u32x4_ptr)(uintptr_t)(uint32_t)addr;
}

struct Prefill64Params {
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
    int tile_tokens;  // kCols / G
    int n_splits;     // key ranges per tile
    int paired;       // tiles of a sequence taken two per workgroup (see prefill_mfma64_plan)
    int rotate;       // the (sequence, KV head) index is rotated by the (tile rank, key range) index (see internal.h)
    int scaled_q;     // the first attempt at a pass works on Q^T times the softmax scale, rounded to bf16 again
    int max_blocks;
    float c;          // softmax_scale * log2(e) (times k_scale for a cache widened from FP8)
    float out_scale;  // multiplies the normalised output: v_scale of an FP8 cache, else 1
};

__global__ __launch_bounds__(kThreads, 1) void prefill64_kernel(Prefill64Params p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- which (pair rank, key split, sequence, KV head) is this workgroup --------------------------------------
    const int n_sg = p.num_seqs * p.hkv_l;
    int item = blockIdx.x;
    const int rank = item / (n_sg * p.n_splits);
    item -= rank * (n_sg * p.n_splits);
    const int split = item / n_sg;
    item -= split * n_sg;
    if (p.rotate) item = (item + n_sg - static_cast<int>((blockIdx.x / n_sg) % n_sg)) % n_sg;
    const int s = item / p.hkv_l;
    const int g = item - s * p.hkv_l;

    const int q_begin = p.cu_seqlens_q[s];
    const int q_len = p.cu_seqlens_q[s + 1] - q_begin;
    const int ctx = p.seq_lens[s];
    const int tile_tokens = p.tile_tokens;
    const int cols_used = tile_tokens * p.G;
    const int n_tiles = (q_len + tile_tokens - 1) / tile_tokens;
    // paired: the workgroup takes tile n_tiles - 1 - rank and then tile rank (heaviest with lightest); else the former
    // alone - workgroups start in the order of their index, so the heaviest tiles of all sequences go first and the light
    // ones fill the compute units that fall free
    const int hi_tile = n_tiles - 1 - rank;
    if (p.paired ? rank > hi_tile : hi_tile < 0) return;  // uniform
    const int n_pass = (!p.paired || hi_tile == rank) ? 1 : 2;
    const_i32_ptr table = (const_i32_ptr)(p.block_table + static_cast<size_t>(s) * p.max_blocks);
    // Inside the key loop the block id of the coming iteration is fetched by a *vector* load: a scalar load shares its
    // counter with the LDS operand reads and returns out of order with them, so while one is outstanding every wait for
    // an operand becomes a wait for everything (measured: 5 % of the kernel).  The address is made to look per-lane
    // (a zero the compiler cannot see through); the id is back in a scalar register by the time the loads need it.
    const int32_t* table_v = p.block_table + static_cast<size_t>(s) * p.max_blocks;
    int lane_zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(lane_zero));
    const int last_block = (ctx - 1) / kBlockSize;

    // in the key loop wavefronts 0 and 1 bring K (cache block 0 / 1 of a tile), wavefronts 2 and 3 V^T
    const bool is_k = wave < 2;
    const int ld_blk = wave & 1;
    const int ld_dst = __builtin_amdgcn_readfirstlane((is_k ? 0 : kKBytes) + ld_blk * kBlockBytes);
    const size_t blk_bytes = static_cast<size_t>(p.hkv_l) * 2 * kBlockBytes;
    // a wavefront-uniform pointer, said explicitly to be in scalar registers
    auto uniform_ptr = [](const unsigned char* ptr) SHIFTATTN_INLINE -> const unsigned char* {
        const uint64_t a = reinterpret_cast<uint64_t>(ptr);
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
        return reinterpret_cast<const unsigned char*>((static_cast<uint64_t>(hi) << 32) | lo);
    };
    const unsigned char* cache_g =
        uniform_ptr(reinterpret_cast<const unsigned char*>(p.cache) + static_cast<size_t>(g) * 2 * kBlockBytes);
    auto block_base = [&](int id) SHIFTATTN_INLINE -> const unsigned char* {
        return cache_g + static_cast<int64_t>(id) * blk_bytes;
    };
    // 4 KiB from src (uniform, scalar registers) + a 32-bit byte offset per lane and load into LDS at dst (uniform).
    // Written as assembly so that the address is formed by the load itself (scalar base + vector offset) instead of a
    // 64-bit vector addition per load.  The LDS destination goes through M0; the compiler treats M0 as reserved (it
    // sets it right before each use of its own and keeps no value in it), so writing it here needs no clobber.  The
    // loads are waited for with explicit vmcnt(0) waits (wait_vm0) only.
    auto dma_4k = [&](const unsigned char* src, const int (&off)[4], unsigned char* dst) SHIFTATTN_INLINE {
        const uint32_t m0v = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(dst));
        asm volatile(
            "s_mov_b32 m0, %0\n\ts_nop 0\n\t"
            "global_load_lds_dwordx4 %1, %5\n\t"
            "global_load_lds_dwordx4 %2, %5 offset:1024\n\t"
            "global_load_lds_dwordx4 %3, %5 offset:2048\n\t"
            "global_load_lds_dwordx4 %4, %5 offset:3072"
            :: "s"(m0v), "v"(off[0]), "v"(off[1]), "v"(off[2]), "v"(off[3]), "s"(src) : "memory");
    };


    for (int pass = 0; pass < n_pass; ++pass) {
        const int tile = pass == 0 ? hi_tile : rank;
        const int tok0 = tile * tile_tokens;
        // ---- LDS addressing (derived from an opaque copy of the lane index in every pass: as loop invariants of the
        // whole kernel these would be kept in registers through the key loop) -------------------------------------
        int lane_p = lane;
        asm volatile("" : "+v"(lane_p));
        const int l32 = lane_p & 31, half = lane_p >> 5;
        const int lds_base = static_cast<int>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) unsigned char*)lds));
        // K operand of MFMA row l32 is K row tau (bits 2 and 3 swapped); piece c of row r sits at c ^ (r & 15)
        const int tau = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
        int k_rd[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) k_rd[ks] = lds_base + tau * 256 + (((2 * ks + half) ^ (tau & 15)) << 4);
        // V^T operand: block-major [2][128 rows][32 B]; the two 16-byte halves of a row are swapped in every other run
        // of eight rows
        const int v_rd = lds_base + kKBytes + l32 * 32 + ((half ^ ((l32 >> 3) & 1)) << 4);
        // Direct-to-LDS loads: one cache block (K or V^T, 4 KiB) per wavefront and iteration as four 1-KiB loads, LDS
        // side contiguous in lane order (the swizzle is applied to the global address).  The loads' immediate offsets
        // (0, 1024, 2048, 3072) move source and destination together, the per-lane offsets carry the rest:
        // K block, load x: rows 4 x + lane / 16, piece lane % 16 of a row stored at (lane % 16) ^ row;
        // V^T block, load x: rows 32 x + lane / 2 (same per-lane offset for every x).
        int k_ld[4];
    #pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int r0 = lane_p >> 4;
            k_ld[x] = r0 * 256 + (((lane_p & 15) ^ r0 ^ (4 * x)) << 4);
        }
        const int v_ld = kBlockBytes + (lane_p >> 1) * 32 + (((lane_p & 1) ^ ((lane_p >> 4) & 1)) << 4);
        int ld_off[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) ld_off[x] = is_k ? k_ld[x] : v_ld;
        int pos_col[2];
        bf16x8 qf[2][8];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int cw = wave * 64 + cb * 32 + l32;
            const int tok = tok0 + cw / p.G;
            const bool valid = cw < cols_used && tok < q_len;
            pos_col[cb] = valid ? ctx - q_len + tok : -1;
        }
        // Q^T of this lane's columns into the accumulation registers.  with_scale: multiplied by the softmax scale (times
        // log2 e, times k_scale of a cache widened from FP8) and rounded to bf16 again, for the attempt that follows no
        // reference: its logits then leave the MFMAs in exp2 units and its loop spends no instruction on scaling them.
        // (the addresses are formed here and not kept: a second fetch is rare)
        auto fetch_q = [&](bool with_scale) SHIFTATTN_INLINE {
            int lane_q = lane;
            asm volatile("" : "+v"(lane_q));
            const uint16_t* q_ptr[2];
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const int cw = wave * 64 + cb * 32 + (lane_q & 31);
                // a column beyond the tile's or the sequence's end reads the row of the nearest real one: every one of
                // its logits is masked (position -1) or its results are dropped, and columns do not mix
                const int cw_r = min(cw, cols_used - 1);
                const int tok_r = min(tok0 + cw_r / p.G, q_len - 1);
                q_ptr[cb] = p.q + static_cast<size_t>(q_begin + tok_r) * p.q_stride + (g * p.G + cw_r % p.G) * kD + (lane_q >> 5) * 8;
            }
            load_q_to_acc(qf[0], qf[1], q_ptr[0], q_ptr[1]);
            if (with_scale) {
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks) {
                        bf16x8 v = qf[cb][ks];
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = static_cast<__bf16>(static_cast<float>(v[e]) * p.c);
                        qf[cb][ks] = v;
                        // (the scaled value is made to look born in accumulation registers, as the loaded one was)
                        asm volatile("" : "+a"(qf[cb][ks]));
                    }
            }
        };
        const int w_tok_first = tok0 + (wave * 64) / p.G;
        const int w_pos_min =
            __builtin_amdgcn_readfirstlane((wave * 64 < cols_used && w_tok_first < q_len) ? ctx - q_len + w_tok_first : -1);

        // ---- key tiles of this (column tile, split) -------------------------------------------------------
        const int tile_pos_max = ctx - q_len + min(tok0 + tile_tokens, q_len) - 1;
        const int kv_tiles = tile_pos_max / kKv + 1;
        const int per_split = (kv_tiles + p.n_splits - 1) / p.n_splits;
        const int kt_begin = __builtin_amdgcn_readfirstlane(split * per_split);
        const int kt_end = min(kv_tiles, kt_begin + per_split);
        const int n = __builtin_amdgcn_readfirstlane(max(kt_end - kt_begin, 0));
        // the tile that reaches past the context (if any) holds unwritten V slots: cleared in LDS before use
        const bool ragged = n > 0 && kt_end * kKv > ctx;

        f32x16 oacc[2][4];
        f32x16 sbuf[2][2];          // [parity][column block]
        u32x4 pw[2][2][2];          // [parity][column block][16-key slice]: four registers of packed P each
        // per column block: reference maximum, its product with the scale (0 while there is none), the largest logit
        // the reference covers (reference + slack), running sum
        float m_used[2] = {-INFINITY, -INFINITY}, mc[2] = {0.f, 0.f}, bound[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
        bool redo = false;          // uniform: a column of this wavefront needed a rescaling the key loop does not do
        float m_rep[2] = {-INFINITY, -INFINITY};
        const float thr = kRefSlack / p.c;  // how far a logit may exceed the reference (attempts that follow the maximum)

        // Ring of three LDS stages: K of tile t and V^T of tile t live in stage t % 3.  Iteration j reads K of tile
        // j + 1 and V^T of tile j - 1 and loads K of tile j + 3 and V^T of tile j + 1, so everything an iteration reads
        // was complete before the barrier of the iteration before: operand reads run on across the barrier.
        int k_cur[8], v_cur;        // LDS addresses of this iteration's operand reads (k_cur[0]: of the next one's)
        int st0 = 0, st1 = 0, st2 = 0;  // byte offsets of stages j % 3, (j + 1) % 3, (j + 2) % 3 at the top of iteration j
        u32x4 pre_a = {0u, 0u, 0u, 0u}, pre_c = pre_a;  // first K and first V^T operand of the coming iteration
        auto next_stage = [](int st) SHIFTATTN_INLINE { return st == 2 * kStageBytes ? 0 : st + kStageBytes; };

        // cache block this wavefront loads in iteration j: K of tile j + 3 or V^T of tile j + 1
        auto load_block_index = [&](int j) SHIFTATTN_INLINE -> int {
            return min(2 * (kt_begin + j + (is_k ? 3 : 1)) + ld_blk, last_block);
        };
        int id_vec = 0;  // block id of the coming iteration's loads, in a vector register until they are issued
        // iterations in which this wavefront loads: K of tiles 3 .. n - 1, V^T of tiles 1 .. n - 1 (a load beyond the last tile
        // would be waited for, with its whole latency, in front of the last product)
        const int ld_limit = n - __builtin_amdgcn_readfirstlane(is_k ? 3 : 1);

        // zero the V^T entries of keys at or past the context in the given stage (tile kt)
        auto clear_ragged_v = [&](int kt, int stage_off) SHIFTATTN_INLINE {
            const int d = tid >> 1, h = tid & 1;
#pragma unroll
            for (int bi = 0; bi < 2; ++bi) {
                const int n_valid = ctx - (kt * kKv + bi * 16 + h * 8);
                if (n_valid < 8) {
                    u32x4* ptr = reinterpret_cast<u32x4*>(lds + stage_off + kKBytes + bi * kBlockBytes + d * 32 +
                                                          ((h ^ ((d >> 3) & 1)) << 4));
                    u32x4 v = *ptr;
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        v[w] &= n_valid > 2 * w + 1 ? 0xFFFFFFFFu : (n_valid > 2 * w ? 0x0000FFFFu : 0u);
                    *ptr = v;
                }
            }
        };

        // One iteration on tile j.  PAR = parity of j: selects the register sets at compile time.
        // TRACK: the tile's maximum is collected and checked against the reference (off only in the steady-state bodies
        // of a pass's first attempt, which check the running sums instead)
        auto body = [&](auto par_c, auto has_a_c, auto has_c_c, auto guard_c, auto track_c, int j) SHIFTATTN_INLINE {
            constexpr int PAR = decltype(par_c)::value;
            // track_c: 1 = the maximum is followed (TRACK); 2 = the reference the column's first key tile left is kept and no
            // maximum followed (KEEP); 0 = no reference at all, on logits that arrive in exp2 units (Q^T carries the scale)
            constexpr bool TRACK = decltype(track_c)::value == 1;
            constexpr bool KEEP = decltype(track_c)::value == 2;
            constexpr bool GUARD = decltype(guard_c)::value != 0;  // outside the steady-state loop
            constexpr bool HAS_A = decltype(has_a_c)::value != 0;
            constexpr bool HAS_C = decltype(has_c_c)::value != 0;
            f32x16(&s_cur)[2] = sbuf[PAR];
            f32x16(&s_nxt)[2] = sbuf[1 - PAR];
            u32x4(&p_cur)[2][2] = pw[PAR];
            u32x4(&p_prv)[2][2] = pw[1 - PAR];
            const int key0 = (kt_begin + j) * kKv;
            // address steps of this iteration: the reads of this iteration's K move on from stage (j+1)%3 to (j+2)%3,
            // those that already serve the next iteration (k_cur[0], v_cur) from (j+2)%3 to (j+3)%3 = j%3
            const int d_now = st2 - st1, d_next = st0 - st2;

            // operand reads: op o feeds the two MFMAs (column blocks 0 and 1) of slots 2 o and 2 o + 1.  Ops beyond this
            // iteration's are the first two of the next one (its first K operand, its first V^T operand).
            constexpr int NOPS = (HAS_A ? 8 : 0) + (HAS_C ? 8 : 0);
            auto read_k = [&](auto ks_c) SHIFTATTN_INLINE -> u32x4 {   // reads with k_cur[ks], then moves it on
                constexpr int ks = decltype(ks_c)::value;
                const u32x4 v = lds_read16(k_cur[ks]);
                k_cur[ks] += ks == 0 ? d_next : d_now;
                asm volatile("" : "+v"(k_cur[ks]));
                return v;
            };
            auto read_v = [&](auto idx_c) SHIFTATTN_INLINE -> u32x4 {
                constexpr int idx = decltype(idx_c)::value;
                return lds_read16(v_cur + (idx / 4) * kBlockBytes + (idx % 4) * 1024);
            };
            auto op_read = [&](auto oc) SHIFTATTN_INLINE -> u32x4 {
                constexpr int o = decltype(oc)::value;
                constexpr bool is_a = HAS_A && (!HAS_C || (o % 2 == 0));
                constexpr int idx = (HAS_A && HAS_C) ? o / 2 : o;
                if constexpr (is_a) return read_k(IC<idx>{});
                else return read_v(IC<idx>{});
            };
            u32x4 opnd[NOPS > 0 ? NOPS : 1];
            if constexpr (NOPS > 0) {
                opnd[0] = HAS_A ? pre_a : pre_c;
                if constexpr (HAS_A && HAS_C) opnd[1] = pre_c;
                else opnd[1] = op_read(IC<1>{});
            }
            if constexpr (!HAS_A) {  // no K reads in this iteration: the addresses move on all the same
#pragma unroll
                for (int ks = 1; ks < 8; ++ks) k_cur[ks] += d_now;
            }
            if constexpr (!HAS_C) v_cur += d_next;

            if (key0 + kKv - 1 > w_pos_min) {  // tile crosses the diagonal of this wavefront: uniform
                // (a real branch: the selects below take their inputs from a statement that cannot be moved out of it)
                asm volatile("; keys beyond a column's position" : "+v"(s_cur[0]), "+v"(s_cur[1]));
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = key0 + 16 * (r >> 3) + 8 * half + (r & 7);
                        if (key > pos_col[cb]) s_cur[cb][r] = -INFINITY;
                    }
            }

            // ---- interleaved block ------------------------------------------------------------------------
            float mx[2] = {-INFINITY, -INFINITY};
            // chunk v (0..31): the logit of column block v / 16, accumulator register v % 16.  Slot v takes the
            // exponential of logit v and finishes logit v - 1 (row sum; on even v the pair (v - 2, v - 1) is packed, on
            // odd v the pair (v - 1, v) enters the maximum): four vector instructions per slot, the exponential
            // counting double, and no instruction uses an exponential issued in its own slot.
            float e_last = 0.f, e_last2 = 0.f;
            auto finish_prev = [&](auto vc) SHIFTATTN_INLINE {  // finishes logit v - 1
                constexpr int v = decltype(vc)::value;
                constexpr int pv = v - 1, cb = pv / 16, r = pv % 16;
                // The row sum runs one logit further behind (logit v - 2): the first vector instruction behind a slot's MFMA
                // then never reads the exponential issued last, which would cost a wait state.
                // (the empty asm statement pins the sum to this slot)
                if constexpr (pv >= 1) {
                    l_run[(pv - 1) / 16] += e_last2;
                    asm volatile("" : "+v"(l_run[(pv - 1) / 16]));
                }
                if constexpr (pv == 31) {
                    l_run[1] += e_last;
                    asm volatile("" : "+v"(l_run[1]));
                }
                if constexpr (r % 2 == 1) {
                    bf16x2 t;
                    t[0] = static_cast<__bf16>(e_last2);
                    t[1] = static_cast<__bf16>(e_last);
                    p_cur[cb][r >> 3][(r & 7) >> 1] = __builtin_bit_cast(uint32_t, t);
                    // (pinned to this slot: left free, the packing drifts together and the slots lose their balance)
                    if constexpr (!TRACK) asm volatile("" : "+v"(p_cur[cb][r >> 3]));
                }
            };
            auto chunk = [&](auto vc) SHIFTATTN_INLINE {
                constexpr int v = decltype(vc)::value;
                constexpr int cb = v / 16, r = v % 16;
                // (no reference followed: Q^T carries the scale, the logit arrives in exp2 units)
                const float e = TRACK        ? __builtin_amdgcn_exp2f(fmaf(s_cur[cb][r], p.c, -mc[cb]))
                                : KEEP       ? __builtin_amdgcn_exp2f(fmaf(s_cur[cb][r], p.c, -mc[cb]))
                                             : __builtin_amdgcn_exp2f(s_cur[cb][r]);
                if constexpr (v >= 1) finish_prev(IC<v>{});
                if constexpr (TRACK && r % 2 == 1) {
                    mx[cb] = fmaxf(fmaxf(mx[cb], s_cur[cb][r - 1]), s_cur[cb][r]);
                    asm volatile("" : "+v"(mx[cb]));
                }
                e_last2 = e_last;
                e_last = e;
                if constexpr (v == 31) finish_prev(IC<32>{});
            };
            auto op_mfma = [&](auto tc, u32x4 a) SHIFTATTN_INLINE {
                constexpr int t = decltype(tc)::value;
                constexpr int o = t / 2, cb = t % 2;
                constexpr bool is_a = HAS_A && (!HAS_C || (o % 2 == 0));
                constexpr int idx = (HAS_A && HAS_C) ? o / 2 : o;
                if constexpr (is_a) {
                    if constexpr (idx == 0) mfma_s_first<GUARD>(s_nxt[cb], a, qf[cb][idx]);
                    else mfma_s_acc<GUARD>(s_nxt[cb], a, qf[cb][idx]);
                } else {
                    constexpr int ks2 = idx / 4, mt = idx % 4;
                    mfma_o_acc<GUARD>(oacc[cb][mt], a, p_prv[cb][ks2]);
                }
            };
            // what runs once per iteration besides the slots: the barrier (with the wait for this wavefront's loads of
            // the iteration before), then the loads into the stages nobody reads any more, then the next block id
            auto fill = [&]() SHIFTATTN_INLINE {
                // a bare barrier: __syncthreads() would first drain every outstanding LDS read.  What has to be complete
                // is this wavefront's loads of the iteration before (waited for here, and with them the block id
                // requested then) and its reads of the stages about to be overwritten (their data went into MFMAs one
                // iteration ago).
                wait_vm0();
                asm volatile("s_barrier" ::: "memory");
                if (j < ld_limit)
                    dma_4k(uniform_ptr(block_base(__builtin_amdgcn_readfirstlane(id_vec))), ld_off, lds + (is_k ? st0 : st1) + ld_dst);
                id_vec = table_v[load_block_index(j + 1) + lane_zero];  // for the loads of the next iteration
            };

            if constexpr (NOPS == 0) {
                fill();
                [&]<int... C>(std::integer_sequence<int, C...>) SHIFTATTN_INLINE { (chunk(IC<C>{}), ...); }
                (std::make_integer_sequence<int, 32>{});
            } else {
                constexpr int kFillSlot = 2;
                [&]<int... T>(std::integer_sequence<int, T...>) SHIFTATTN_INLINE {
                    (([&]() SHIFTATTN_INLINE {
                         constexpr int o = T / 2;
                         if constexpr (T % 2 == 0) {
                             if constexpr (o + 2 < NOPS) {
                                 opnd[o + 2] = op_read(IC<o + 2>{});
                                 // the V^T base moves on once this iteration's last V^T operand is requested
                                 if constexpr (HAS_C && o + 2 == NOPS - 1) {
                                     v_cur += d_next;
                                     asm volatile("" : "+v"(v_cur));
                                 }
                             } else if constexpr (o + 2 == NOPS) {
                                 pre_a = read_k(IC<0>{});
                             } else {
                                 pre_c = read_v(IC<0>{});
                             }
                         }
                         op_mfma(IC<T>{}, opnd[o]);
                         __builtin_amdgcn_sched_barrier(0);  // the softmax work of the slot goes behind its MFMA
                         if constexpr (T == kFillSlot) fill();
                         if constexpr (NOPS == 16) {
                             chunk(IC<T>{});
                         } else {
                             chunk(IC<2 * T>{});
                             chunk(IC<2 * T + 1>{});
                         }
                         __builtin_amdgcn_sched_barrier(0);
                     }()),
                     ...);
                }
                (std::make_integer_sequence<int, 2 * NOPS>{});
            }

            // ---- the tile's maximum against what the reference covers: rarely, a new reference ------------------
            if constexpr (TRACK)
            if (__builtin_expect(__builtin_amdgcn_ballot_w64(mx[0] > bound[0] || mx[1] > bound[1]) != 0, 0)) {
                // A column that meets its first visible keys has no sums yet (O^T = 0, l = 0): its reference is set and
                // the tile's P recomputed, nothing else.  A column that already holds sums would need them rescaled;
                // O^T is not touched by the vector ALU inside this loop (that would pull it out of the accumulation
                // registers), so such a tile only flags the pass, which is then run a second time from the reference
                // this attempt ends with.
                bool bad = false;
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    // both lanes of a column (its two halves of the keys) must take the same decision
                    const float mo = __shfl_xor(mx[cb], 32);
                    const float mfull = fmaxf(mx[cb], mo);
                    const bool grow = mfull > bound[cb];
                    bad = bad || (grow && m_used[cb] != -INFINITY);
                    if (grow) {
                        m_used[cb] = mfull;
                        mc[cb] = mfull * p.c;
                        bound[cb] = mfull + thr;
                    }
                    float ps = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        const float e0 = __builtin_amdgcn_exp2f(fmaf(s_cur[cb][r], p.c, -mc[cb]));
                        const float e1 = __builtin_amdgcn_exp2f(fmaf(s_cur[cb][r + 1], p.c, -mc[cb]));
                        bf16x2 t;
                        t[0] = static_cast<__bf16>(e0);
                        t[1] = static_cast<__bf16>(e1);
                        ps += e0;
                        ps += e1;
                        p_cur[cb][r >> 3][(r & 7) >> 1] = __builtin_bit_cast(uint32_t, t);
                    }
                    if (grow) l_run[cb] = ps;  // (a column that keeps its reference has just recomputed what it had)
                }
                if (__builtin_amdgcn_ballot_w64(bad)) redo = true;
            }
            const int st_new = st0;  // (j + 3) % 3
            st0 = st1;
            st1 = st2;
            st2 = st_new;
        };

        // prologue loads: K of the first three tiles and V^T of the first (two cache blocks per wavefront)
        auto issue_prologue = [&]() SHIFTATTN_INLINE {
            const int id_p = table[min(2 * (kt_begin + (wave >> 1)) + ld_blk, last_block)];
            dma_4k(uniform_ptr(block_base(id_p)), k_ld, lds + (wave >> 1) * kStageBytes + ld_blk * kBlockBytes);
            // the loads "iteration -1" would have issued: K of tile 2 into stage 2, V^T of tile 0 into stage 0
            const int id_q = table[load_block_index(-1)];
            dma_4k(uniform_ptr(block_base(id_q)), ld_off, lds + (is_k ? 2 * kStageBytes : 0) + ld_dst);
            id_vec = table_v[load_block_index(0) + lane_zero];
        };
        // The first attempt's go out in front of the fetch of Q^T, whose wait then covers both.
        if (n > 0) issue_prologue();
        fetch_q(p.scaled_q != 0);

        // Up to three attempts at the pass.  The first follows no maximum behind the first key tile (its steady-state
        // bodies save the instruction per two logits that would collect it; real logits stay within 2^100 of their
        // first tile's maximum).  If some wavefront flags it (see the end of an iteration), the second starts over and
        // follows the maximum tile by tile; it can end flagged itself (a column outgrew its reference after it had sums),
        // and then holds, for every column, a reference within the slack of the true maximum: the third attempt starts
        // from that and is not flagged.
        for (int attempt = 0; attempt < 3; ++attempt) {
        redo = false;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            l_run[cb] = 0.f;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[cb][mt][r] = 0.f;
        }
        auto key_loop = [&](auto track_c) SHIFTATTN_INLINE {
            // prologue: the loads (already on their way in the first attempt), S^T of the first tile
            if (attempt > 0) issue_prologue();
            st0 = 0, st1 = kStageBytes, st2 = 2 * kStageBytes;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) k_cur[ks] = k_rd[ks] + kStageBytes;   // iteration 0 reads K of tile 1
            v_cur = v_rd + 2 * kStageBytes;                                       // (nothing; iteration 1 reads stage 0)
            wait_vm0();
            __syncthreads();
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const u32x4 a = lds_read16(k_rd[ks]);
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    if (ks == 0) mfma_s_first<true>(sbuf[0][cb], a, qf[cb][ks]);
                    else mfma_s_acc<true>(sbuf[0][cb], a, qf[cb][ks]);
                }
            }
            pre_a = lds_read16(k_cur[0]);
            k_cur[0] += kStageBytes;  // on to stage 2: iteration 1's first K operand
            mfma_settle();
            // (the attempt that keeps its first tile's reference takes it here, from a tile that follows the maximum)
            constexpr int kFirst = decltype(track_c)::value == 2 ? 1 : decltype(track_c)::value;
            if (n == 1) {
                body(IC<0>{}, IC<0>{}, IC<0>{}, IC<1>{}, IC<kFirst>{}, 0);
            } else {
                body(IC<0>{}, IC<1>{}, IC<0>{}, IC<1>{}, IC<kFirst>{}, 0);
                int j = 1;  // stays odd: the steady-state loop takes two tiles per trip so that the register sets of
                            // even and odd tiles are fixed at compile time
                for (; j + 2 < n; j += 2) {
                    body(IC<1>{}, IC<1>{}, IC<1>{}, IC<0>{}, track_c, j);
                    body(IC<0>{}, IC<1>{}, IC<1>{}, IC<0>{}, track_c, j + 1);
                }
                if (j + 1 < n) {
                    body(IC<1>{}, IC<1>{}, IC<1>{}, IC<1>{}, track_c, j);
                    body(IC<0>{}, IC<0>{}, IC<1>{}, IC<1>{}, track_c, j + 1);
                } else {
                    body(IC<1>{}, IC<0>{}, IC<1>{}, IC<1>{}, track_c, j);
                }
            }
            // epilogue: O^T += V^T P^T of the last tile (tile n - 1, in stage (n - 1) % 3 = st2 by now)
            wait_vm0();
            __syncthreads();
            const int lp = (n - 1) & 1;
            if (ragged) {
                clear_ragged_v(kt_begin + n - 1, st2);
                __syncthreads();
            }
            auto last_c = [&](auto par_c) SHIFTATTN_INLINE {
                constexpr int PAR = decltype(par_c)::value;
#pragma unroll
                for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt) {
                        const u32x4 a = lds_read16(st2 + v_rd + ks2 * kBlockBytes + mt * 1024);
#pragma unroll
                        for (int cb = 0; cb < 2; ++cb) {
                            mfma_o_acc<true>(oacc[cb][mt], a, pw[PAR][cb][ks2]);
                        }
                    }
            };
            if (lp) last_c(IC<1>{});
            else last_c(IC<0>{});
            mfma_settle();
        };
        if (n > 0) {
            if (attempt > 0) key_loop(IC<1>{});
            else if (p.scaled_q) key_loop(IC<0>{});
            else key_loop(IC<2>{});
        }
        if (attempt == 0) {
            // The first attempt followed no maximum.  That is exact as long as nothing left the range bf16 and the fp32 sums
            // hold without loss.  With the first tile's reference kept: a column's sum must not exceed 2^100 (P then stays
            // below it; what underflows is negligible beside the first tile's keys).  With no reference at all: a column that
            // sees keys of this range must end with a sum inside [2^-40, 2^40].  An infinity or a NaN fails either test; the
            // pass is then flagged.
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const float l_tot = l_run[cb] + __shfl_xor(l_run[cb], 32);
                if (p.scaled_q) {
                    const bool sees = n > 0 && pos_col[cb] >= kt_begin * kKv;
                    if (sees && !(l_tot >= kFreeSumLo && l_tot <= kFreeSumHi)) redo = true;
                    m_rep[cb] = sees ? 0.f : -INFINITY;   // what a partial result reports as its reference (exp2 units)
                } else {
                    if (!(l_tot <= kKeepSumBound)) redo = true;
                    m_rep[cb] = m_used[cb] * p.c;
                }
            }
            redo = __builtin_amdgcn_ballot_w64(redo) != 0;
        } else {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) m_rep[cb] = m_used[cb] * p.c;
        }
        if (attempt == 2) break;
        int* flags = reinterpret_cast<int*>(lds + kRingBytes + kCols * kPitch);
        if (lane == 0) flags[wave] = redo ? 1 : 0;
        __syncthreads();  // also: every wavefront is done with the ring
        const int any_redo = flags[0] | flags[1] | flags[2] | flags[3];
        if (__builtin_expect(__builtin_amdgcn_readfirstlane(any_redo) == 0, 1)) break;
        if (attempt == 0) {   // the attempts that follow the maximum start without references, on Q^T as given
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) m_used[cb] = -INFINITY, mc[cb] = 0.f, bound[cb] = -INFINITY;
            if (p.scaled_q) fetch_q(false);
        }
        }

        // ---- results of the pass ----------------------------------------------------------------------------
        // the lane index is read through an opaque copy: addresses derived from the plain value are loop invariants
        // that the optimiser computes before the key loop and then keeps in registers through it
        int lane_m = lane;
        asm volatile("" : "+v"(lane_m));
        const int l32_m = lane_m & 31, half_m = lane_m >> 5;
        if (p.n_splits == 1) {
            // normalise, put bf16 rows into this wavefront's part of the staging tile, then write them out in whole
            // 256-byte rows (one 16-byte piece per lane, 1 KiB of consecutive output per 4 rows)
            unsigned char* stage = lds + kRingBytes + wave * 64 * kPitch;
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const float l_tot = l_run[cb] + __shfl_xor(l_run[cb], 32);
                const float inv = l_tot > 0.f ? p.out_scale / l_tot : 0.f;
                unsigned char* srow = stage + (cb * 32 + l32_m) * kPitch + 8 * half_m;
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        // accumulator register r of row tile mt is head-dim 32*mt + 8*(r/4) + 4*half + r%4
                        bf16x4 v;
#pragma unroll
                        for (int x = 0; x < 4; ++x) v[x] = static_cast<__bf16>(oacc[cb][mt][r4 * 4 + x] * inv);
                        *reinterpret_cast<u32x2*>(srow + (32 * mt + 8 * r4) * 2) = __builtin_bit_cast(u32x2, v);
                    }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int col = 4 * i + (lane_m >> 4), piece = lane_m & 15;
                const int cw = wave * 64 + col;
                const int tok_c = tok0 + cw / p.G;
                if (cw < cols_used && tok_c < q_len) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(stage + col * kPitch + piece * 16);
                    uint16_t* op = p.out + static_cast<size_t>(q_begin + tok_c) * p.out_stride + (g * p.G + cw % p.G) * kD + piece * 8;
                    *reinterpret_cast<u32x4*>(op) = v;
                }
            }
        } else {
            // key ranges split over workgroups: the un-normalised partial of this range
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const float l_tot = l_run[cb] + __shfl_xor(l_run[cb], 32);
                if (pos_col[cb] >= 0) {
                    const int cw = wave * 64 + cb * 32 + l32_m;
                    const int row_col = q_begin + tok0 + cw / p.G;
                    const int head_col = g * p.G + cw % p.G;
                    const size_t prow = (static_cast<size_t>(split) * p.total_q + row_col) * p.hq_l + head_col;
                    float* op = p.o_part + prow * kD + 4 * half_m;
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            f32x4 v;
#pragma unroll
                            for (int x = 0; x < 4; ++x) v[x] = oacc[cb][mt][r4 * 4 + x];
                            *reinterpret_cast<f32x4*>(op + 32 * mt + 8 * r4) = v;
                        }
                    if (half_m == 0) {
                        p.ml_part[prow * 2] = m_rep[cb];  // exp2 units; -inf when this key range held no visible key
                        p.ml_part[prow * 2 + 1] = l_tot;
                    }
                }
            }
        }
        // The next pass reuses the ring, the flags and the staging tile: every wavefront must have left this pass's last
        // LDS reads behind.  A bare barrier: __syncthreads() would also wait for the output stores just issued (several
        // microseconds until the last is acknowledged); nothing in the next pass depends on them, and its first loads
        // overlap them.
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
}

}  // namespace

bool prefill_mfma64_supported(const AttnShape& a) {
    return a.elem == 2 && a.D == kD && !a.kv_fp8() && a.hq_l % a.hkv_l == 0 && a.hq_l / a.hkv_l <= kCols;
}

Prefill64Plan prefill_mfma64_plan(int num_seqs, int total_q, int max_q_len, int max_seq_len, const AttnShape& a,
                                  int forced_splits) {
    Prefill64Plan pl;
    const int G = a.hq_l / a.hkv_l;
    pl.tile_tokens = kCols / G;
    const int tiles = (max_q_len + pl.tile_tokens - 1) / pl.tile_tokens;
    // Causal tiles differ in work (tile i sees i + 1 tiles' worth of keys).  Two ways to level it: a workgroup takes the
    // heaviest tile left together with the lightest (equal workgroups, one round when the pairs fit the chip), or one
    // tile per workgroup, heaviest first, the light ones filling the compute units that fall free (any number of tiles
    // levels out, but a tile is never shorter than its keys: it wants key ranges when the heaviest outweighs a compute
    // unit's share).  A short chunk behind a long context has nothing to level - its tiles all walk the context - and
    // pairing only makes every workgroup pay set-up, first tile and write-out twice.  Both are priced with the same rough
    // model (plus kPassSeconds per pass a compute unit makes) over the key ranges per tile - a workgroup's time falls with
    // the ranges, every range adds a partial result per (token, head) that the merge kernel writes and reads back - and
    // the cheaper plan is taken.
    constexpr double kPassSeconds = 15e-6;  // set-up, Q fetch, first and last tiles, write-out: what a pass costs around its loop
    const double seqs_equiv = longest_chunk_equivalents(num_seqs, total_q, max_q_len);
    const int by_len = max_seq_len / (32 * kKv);  // at least 32 key tiles per range
    struct Cand {
        int splits;
        double seconds, with_passes;
    };
    auto best_of = [&](auto model) {  // model(splits) -> {seconds, passes per compute unit}
        Cand best = {0, 0.0, 0.0};
        auto take = [&](int sp) {
            const auto [t, passes] = model(sp);
            const Cand c = {sp, t, t + passes * kPassSeconds};
            if (best.splits == 0 || c.with_passes < best.with_passes * 0.97) best = c;  // a further range must pay for itself
        };
        if (forced_splits > 0) take(forced_splits);
        else
            for (int cand = 1; cand <= 16 && (cand == 1 || cand <= by_len); ++cand) take(cand);
        return best;
    };
    const int pair_ranks = (tiles + 1) / 2;
    const Cand paired = best_of([&](int sp) {
        const long wgs = static_cast<long>(pair_ranks) * num_seqs * a.hkv_l;
        const double rounds = static_cast<double>((wgs * sp + 255) / 256);
        return std::pair<double, double>(
            launch_model_seconds(wgs, sp, kCols, total_q, max_seq_len, a.hq_l, paired_walks(max_q_len, max_seq_len)), 2.0 * rounds);
    });
    const Cand single = best_of([&](int sp) {
        // tile i of a sequence walks (S - Q + (i + 1) tile_tokens) / S of the longest context S
        const double S = max_seq_len > 0 ? max_seq_len : 1, Q = max_q_len < max_seq_len ? max_q_len : max_seq_len;
        const double unit = 4.0 * 128 * kCols * S / 3.9e12, merge = 2.0 * total_q * a.hq_l * 130 * 4 / 4.0e12;
        const double base = (S - Q) / S, step = pl.tile_tokens / S;
        const double seqs = seqs_equiv;
        const double total = (tiles * base + step * tiles * (tiles + 1) / 2.0) * seqs * a.hkv_l;
        const double heaviest = (base + step * tiles < 1.0 ? base + step * tiles : 1.0) / sp;
        const long items = static_cast<long>(tiles * seqs * a.hkv_l * sp + 0.5);
        const double share = 1.03 * total / 256.0;  // a compute unit's share of all the work, filled by ever lighter tiles
        const double span = items <= 256 ? heaviest : (heaviest > share ? heaviest : share);
        return std::pair<double, double>(span * unit + (sp > 1 ? sp * merge + 5.0e-6 : 0.0), static_cast<double>((items + 255) / 256));
    });
    const int forced_pairing = option_prefill_pairing();
    pl.paired = forced_pairing == 1 || (forced_pairing == 0 && paired.with_passes <= single.with_passes);
    pl.pair_ranks = pl.paired ? pair_ranks : tiles;
    int splits = pl.paired ? paired.splits : single.splits;
    pl.model_seconds = pl.paired ? paired.seconds : single.seconds;
    pl.model_with_passes = pl.paired ? paired.with_passes : single.with_passes;
    if (splits < 1) splits = 1;
    if (splits > 64) splits = 64;
    pl.n_splits = splits;
    pl.rotate = rotate_sequences_over_dies(num_seqs, a.hkv_l, total_q, max_q_len);
    pl.workgroups = static_cast<long>(pl.pair_ranks) * splits * num_seqs * a.hkv_l;
    return pl;
}

size_t prefill_mfma64_workspace(int total_q, const Prefill64Plan& pl, const AttnShape& a) {
    return pl.n_splits == 1 ? 0 : static_cast<size_t>(pl.n_splits) * total_q * a.hq_l * (kD + 2) * sizeof(float);
}

hipError_t prefill_mfma64_init() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill64_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               kLdsBytes);
}

hipError_t launch_prefill_mfma64(const void* q, const void* cache, const int32_t* block_table, int max_blocks,
                                 const int32_t* cu_seqlens_q, const int32_t* seq_lens, int num_seqs, int total_q,
                                 const Prefill64Plan& pl, void* out, void* workspace, const AttnShape& a, float c,
                                 float out_scale, hipStream_t st) {
    Prefill64Params p;
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
    p.tile_tokens = pl.tile_tokens;
    p.n_splits = pl.n_splits;
    p.paired = pl.paired ? 1 : 0;
    p.rotate = pl.rotate ? 1 : 0;
    p.scaled_q = option_prefill_scaled_q() ? 1 : 0;
    p.max_blocks = max_blocks;
    p.c = c;
    p.out_scale = out_scale;
    prefill64_kernel<<<static_cast<unsigned>(pl.workgroups), kThreads, kLdsBytes, st>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (pl.n_splits > 1)
        return launch_combine(p.o_part, p.ml_part, total_q, a.hq_l, kD, pl.n_splits, 0, nullptr, 0, out, a.out_stride, a.elem,
                              out_scale, st);
    return hipSuccess;
}

}  // namespace shiftattn
