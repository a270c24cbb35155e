// Paged decode attention, split over the context (Algorithm 1 boxed line for decode rows; the
// paper's observation that decoding re-reads the whole KV cache per token and ends up bound by
// memory bandwidth, Sec. 4.3).  bf16 cache, head_dim 128, up to 16 query heads per KV head.
//
// A wavefront works through its tokens in 32-token groups (two cache blocks).  All query heads of the GQA
// group ride in the 16-wide N dimension of a 16x16x32 bf16 MFMA, so every K and V byte is read from HBM
// once per (sequence, KV head) and used for all heads:
//   S^T[token][head]  = K[token][:] . Q^T[:][head]        A = K rows,   B = Q^T (registers)
//   O^T[d][head]     += V^T[d][token] . P^T[token][head]   A = V^T rows, B = P^T (from S^T regs)
// K is stored token-major and V dimension-major in the cache, so both A operands are contiguous
// 16-byte pieces.  Tokens are assigned to MFMA rows so that the eight S^T values a lane holds
// (two 16-token tiles x four rows) are eight consecutive tokens: exactly the k-slice of P^T the
// second MFMA needs from that lane, and exactly one 16-byte piece of a V^T row.
//
// Partial results are un-normalised (max, sum, O) per head; the merge kernel folds the parts of a row in
// part order, so results do not depend on scheduling.
//
// Decomposition: decode_flat_kernel lays all (sequence, KV head) pairs end to end, each padded to a
// multiple of 32 tokens, and gives every wavefront of a fixed-size grid the same number of tokens of
// that line, whatever the mix of context lengths: all wavefronts start and finish together, none waits
// at a barrier, and a wavefront pays its start-up latency once.  A wavefront emits one partial per
// sequence its range touches; sorted by position these partials are numbered (wavefront index + pair
// index), so the parts of a pair are consecutive rows.  The kernel indexes up to 2048 pairs in LDS; a
// larger batch is served in runs of that many pairs, one launch (and one merge) per run.
//
// Appending the new token (flat kernel): when the call brings the new tokens' K/V, the wavefront whose
// range holds the last group of a (sequence, KV head) pair stores that pair's new K row and V column into
// the cache itself and overwrites them in its parked copy of the group, so the result is the one of
// "append, then attend" without a separate launch in front.  The slot of a sequence's new token must be
// the slot of its position seq_lens - 1 (the append a decode step performs).
//
// FP8 E4M3 cache (flat kernel only): a cache block is half as many bytes in the same arrangement, so a
// group takes eight 1-KiB loads instead of sixteen; every loaded 16-byte piece (16 codes) is widened in
// registers to the two bf16 pieces it stands for (exact: every E4M3 value is a bf16 value) and parked
// where the bf16 path would have put them, so the LDS layout, the operand reads and all arithmetic are
// shared.  k_scale rides in the logit scale, v_scale in the merge.
#include "internal.h"

#include <stdlib.h>

namespace shiftattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kWaves = 4;
constexpr int kGroup = 32;         // tokens per wavefront step
constexpr int kOPad = kD + 4;      // LDS row pitch (floats) of the per-wavefront O staging

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct GroupFrags {
    u32x4 k[8];  // [tile a/b][4 head-dim steps]
    u32x4 v[8];  // [8 row tiles of 16 head-dim rows]
};

// Memory access: every load instruction of a wavefront covers 1 KiB of consecutive bytes of a cache
// block (non-temporal), so each 128-byte line is requested exactly once and the L1 sees eight whole
// lines per instruction (loading straight in MFMA operand layout would touch sixteen half lines per
// instruction and measured ~15 % slower).  The pieces are parked in a wavefront-private, XOR-swizzled
// LDS area and the MFMA operands are read back from there without bank conflicts; the next group's
// loads are already in flight in registers meanwhile.
constexpr int kStageBytes = 16384;  // per wavefront: K of two blocks (2 x 4 KiB), V^T of two blocks (2 x 4 KiB)

constexpr int kFlatMaxPairs = 2048;                       // (sequence, KV head) pairs indexed in LDS
constexpr int kFlatWorkgroups = 512;                      // two resident per compute unit
constexpr int kFlatWorkers = kFlatWorkgroups * kWaves;    // wavefronts, each with its own token range

// The flat kernel: see the file header.  cum[i + 1] holds the padded token count of pairs 0..i in
// its upper bits and (padded - real) length of pair i in its low five bits.
// the two bf16 pieces (8 elements each) of one 16-byte piece of E4M3 codes
__device__ inline void widen_fp8(u32x4 codes, u32x4& lo, u32x4& hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        lo[2 * w] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(codes[w]), 1.0f, false));
        lo[2 * w + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(codes[w]), 1.0f, true));
        hi[2 * w] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(codes[2 + w]), 1.0f, false));
        hi[2 * w + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(codes[2 + w]), 1.0f, true));
    }
}

struct AppendArgs {
    const uint16_t* k_new;   // [num_seqs][hkv_l][D] bf16, row stride kv_stride elements
    const uint16_t* v_new;
    const int64_t* slots;    // [num_seqs]; negative: nothing to append for that sequence
    int64_t kv_stride;
    float k_scale, v_scale;  // FP8 cache only
};

template <bool kFp8, bool kAppend>
__global__ __launch_bounds__(kWaves * 64, 2) void decode_flat_kernel(
    const uint16_t* __restrict__ q, int64_t q_stride, uint16_t* __restrict__ cache,
    const int32_t* __restrict__ block_table, int max_blocks, const int32_t* __restrict__ seq_lens,
    float* __restrict__ o_part, float* __restrict__ ml_part, int2* __restrict__ plan, int num_seqs, int hq_l, int hkv_l,
    float c, int r_min, AppendArgs ap) {
    __shared__ __attribute__((aligned(16))) unsigned char smem[kWaves * kStageBytes];
    __shared__ int cum[kFlatMaxPairs + 1];
    __shared__ int wave_sum[kWaves];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int n_pairs = num_seqs * hkv_l;
    const int G = hq_l / hkv_l;

    // ---- padded prefix sums of the context lengths: thread t owns pairs 8t .. 8t+7 -----------------
    {
        constexpr int kPer = kFlatMaxPairs / (kWaves * 64);  // 8
        int len[kPer], pad[kPer];
        int mine = 0;
#pragma unroll
        for (int x = 0; x < kPer; ++x) {
            const int i = threadIdx.x * kPer + x;
            len[x] = i < n_pairs ? max(seq_lens[i / hkv_l], 0) : 0;
        }
#pragma unroll
        for (int x = 0; x < kPer; ++x) {
            pad[x] = (len[x] + kGroup - 1) & ~(kGroup - 1);
            mine += pad[x];
        }
        // inclusive scan over the wavefront with cross-lane moves (rows of 16, then row to row)
        int incl = mine;
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x111, 0xf, 0xf, false);  // row_shr:1
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x112, 0xf, 0xf, false);  // row_shr:2
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x114, 0xf, 0xf, false);  // row_shr:4
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x118, 0xf, 0xf, false);  // row_shr:8
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x142, 0xa, 0xf, false);  // lane 15 of a row into rows 1 and 3
        incl += __builtin_amdgcn_update_dpp(0, incl, 0x143, 0xc, 0xf, false);  // lane 31 into rows 2 and 3
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        int run = incl - mine;
#pragma unroll
        for (int w = 0; w < kWaves; ++w)
            if (w < wave) run += wave_sum[w];
#pragma unroll
        for (int x = 0; x < kPer; ++x) {
            const int i = threadIdx.x * kPer + x;
            run += pad[x];
            if (i < n_pairs) cum[i + 1] = run | (pad[x] - len[x]);
        }
        if (threadIdx.x == 0) cum[0] = 0;
        __syncthreads();
    }
    const int total = __builtin_amdgcn_readfirstlane(cum[n_pairs]) & ~(kGroup - 1);
    int R = ((total + kFlatWorkers - 1) / kFlatWorkers + kGroup - 1) & ~(kGroup - 1);
    R = max(R, r_min);
    if (blockIdx.x == 0) {  // which partial rows belong to which pair, for the merge kernel
        for (int i = threadIdx.x; i < n_pairs; i += kWaves * 64) {
            const int a = cum[i] & ~(kGroup - 1), b = cum[i + 1] & ~(kGroup - 1);
            int2 e = {0, 0};
            if (b > a) {
                const int w0 = a / R, w1 = (b - 1) / R;
                e.x = w0 + i;
                e.y = w1 - w0 + 1;
            }
            plan[i] = e;
        }
    }
    const int wk = blockIdx.x * kWaves + wave;
    const int64_t start64 = static_cast<int64_t>(wk) * R;
    if (start64 >= total) return;  // no barrier below this line
    const int start = static_cast<int>(start64);
    const int end = min(start + R, total);

    const int col = lane & 15;
    const int grp = lane >> 4;
    unsigned char* my = smem + wave * kStageBytes;
    // LDS layout of a parked group (per wavefront, 16-byte pieces).  K of block b (4 KiB at 4096 b): row t at
    // 256 t, piece p of the row stored at column p ^ (t & 3) ^ 4 ((t >> 2) ^ b); load j of a block brings rows
    // 4 j + lane / 16, piece lane % 16.  V^T of block b (4 KiB at 8192 + 4096 b): piece 64 j + lane of load j
    // (row 32 j + lane / 2, half lane % 2) stored with its low bit flipped in every other run of 16 pieces.
    // K operand: token row tau (+4 for tile b) of block k_sel, piece grp + 4 kk; V^T operand: piece
    // 2 (16 mt + col) + grp % 2 of block grp / 2.  The positions are folded so that four bases serve the K
    // writes, four the K reads and one each the V^T writes and reads; the rest are immediate offsets.
    //   K write, block b, load j   : kw[j ^ b] + 4096 b + 1024 j
    //   K read, tile a / b, step kk: kr[kk] / kr[kk ^ 1] + 1024
    int kw[4], kr[4];
    {
        const int r0 = lane >> 4, p = lane & 15;
        const int base = r0 * 256 + ((p ^ r0) << 4);
        const int tau_a = ((col >> 2) << 3) + (col & 3);
        const int k_sel = tau_a >> 4, k_off_a = tau_a & 15;
        const int rbase = k_sel * 4096 + k_off_a * 256 + ((grp ^ k_off_a ^ (4 * k_sel)) << 4);
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            kw[x] = base ^ (64 * x);
            kr[x] = rbase ^ (64 * x);
        }
    }
    const int vw = 8192 + ((lane ^ ((lane >> 4) & 1)) << 4);
    const int vr = 8192 + (grp >> 1) * 4096 + (((2 * col + (grp & 1)) ^ ((col >> 3) & 1)) << 4);
    // FP8 cache: a 1-KiB load covers eight K rows (lane >> 3) of eight 16-code pieces (lane & 7), or 64 V^T
    // rows (lane) of one piece.  Piece q (0 / 1) of the widened pair goes to
    //   K, block b, load j  : (kw8 ^ 64 (2j ^ b) ^ 16 q) + 4096 b + 2048 j     (same swizzle as above, row 8j + lane/8)
    //   V^T, block b, load j: (vw8 ^ 16 q) + 4096 b + 2048 j
    int kw8 = 0, vw8 = 0;
    if constexpr (kFp8) {
        const int r8 = lane >> 3, pc = lane & 7;
        kw8 = r8 * 256 + (((2 * pc) ^ (r8 & 3) ^ (4 * (lane >> 5))) << 4);
        const int l31 = lane & 31;
        vw8 = 8192 + 1024 * (lane >> 5) + (((2 * l31) ^ ((l31 >> 3) & 1)) << 4);
    }

    // ---- a position on the line: pair index, its padded token range, its real length (all scalar) --
    int pos = start, pair, seg_begin, seg_end, ctx;
    auto seg_of = [&](int pr, int& sb, int& se, int& cx) {
        const int lo = __builtin_amdgcn_readfirstlane(cum[pr]);
        const int hi = __builtin_amdgcn_readfirstlane(cum[pr + 1]);
        sb = lo & ~(kGroup - 1);
        se = hi & ~(kGroup - 1);
        cx = se - sb - (hi & (kGroup - 1));
    };
    {
        // first pair whose padded range ends beyond `start` (one exists: start < total): every lane
        // probes one entry, first among 64 evenly spaced ones, then inside the stretch that brackets it
        const int step = (n_pairs + 63) / 64;
        const int probe = min((lane + 1) * step, n_pairs);
        const uint64_t coarse = __builtin_amdgcn_ballot_w64((cum[probe] & ~(kGroup - 1)) > start);
        const int base = __builtin_ctzll(coarse) * step;  // the answer lies in [base, base + step)
        int lo = base;
        for (int b = base; b < base + step; b += 64) {
            const int i = min(b + lane, n_pairs - 1);
            const uint64_t fine = __builtin_amdgcn_ballot_w64((cum[i + 1] & ~(kGroup - 1)) > start);
            if (fine) {
                lo = b + __builtin_ctzll(fine);
                break;
            }
        }
        pair = __builtin_amdgcn_readfirstlane(lo);
        seg_of(pair, seg_begin, seg_end, ctx);
    }
    // block ids of the group at (pr, ps); scalar loads
    auto fetch_ids = [&](int pr, int ps, int sb, int cx, int& blk0, int& blk1) {
        const int s = pr / hkv_l;
        const int b0 = (ps - sb) / kBlockSize;
        const int last_block = (cx - 1) / kBlockSize;
        const int32_t* table = block_table + static_cast<size_t>(s) * max_blocks;
        blk0 = table[b0];
        blk1 = table[min(b0 + 1, last_block)];
    };
    GroupFrags f;
    auto load_group = [&](int pr, int blk0, int blk1) {
        const int g = pr % hkv_l;
        if constexpr (kFp8) {  // one byte per element: K 2 KiB then V^T 2 KiB per (block, head)
            const unsigned char* cb = reinterpret_cast<const unsigned char*>(cache);
            const u32x4* k0 = reinterpret_cast<const u32x4*>(cb + cache_part_offset(blk0, g, 0, hkv_l, kD)) + lane;
            const u32x4* k1 = reinterpret_cast<const u32x4*>(cb + cache_part_offset(blk1, g, 0, hkv_l, kD)) + lane;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                f.k[j] = __builtin_nontemporal_load(k0 + 64 * j);
                f.k[2 + j] = __builtin_nontemporal_load(k1 + 64 * j);
                f.v[j] = __builtin_nontemporal_load(k0 + 128 + 64 * j);
                f.v[2 + j] = __builtin_nontemporal_load(k1 + 128 + 64 * j);
            }
        } else {
            const u32x4* k0 = reinterpret_cast<const u32x4*>(cache + cache_part_offset(blk0, g, 0, hkv_l, kD)) + lane;
            const u32x4* k1 = reinterpret_cast<const u32x4*>(cache + cache_part_offset(blk1, g, 0, hkv_l, kD)) + lane;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f.k[j] = __builtin_nontemporal_load(k0 + 64 * j);
                f.k[4 + j] = __builtin_nontemporal_load(k1 + 64 * j);
                f.v[j] = __builtin_nontemporal_load(k0 + 256 + 64 * j);
                f.v[4 + j] = __builtin_nontemporal_load(k1 + 256 + 64 * j);
            }
        }
    };
    bf16x8 qf[4];
    auto load_q = [&](int pr) {
        const int s = pr / hkv_l, g = pr % hkv_l;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (col < G)
                v = *reinterpret_cast<const u32x4*>(q + static_cast<size_t>(s) * q_stride +
                                                    static_cast<size_t>(g * G + col) * kD + 8 * (grp + 4 * kk));
            qf[kk] = as_bf16x8(v);
        }
    };

    f32x4 o[8];
    float m_run, l_run;
    auto reset = [&]() {
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) o[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        m_run = -INFINITY;
        l_run = 0.f;
    };
    auto flush = [&](int pr) {  // this wavefront's partial of pair `pr`: row (wavefront + pair)
        float l = l_run + __shfl_xor(l_run, 16);
        l += __shfl_xor(l, 32);
        if (col < G) {
            const size_t prow = (static_cast<size_t>(wk) + pr) * G + col;
            float* dst = o_part + prow * kD + 4 * grp;
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) *reinterpret_cast<f32x4*>(dst + 16 * mt) = o[mt];
            if (grp == 0) {
                ml_part[prow * 2] = m_run * c;
                ml_part[prow * 2 + 1] = l;
            }
        }
    };

    // ---- pipeline: while group i is computed from LDS, the loads of group i+1 are in flight (into the
    // registers group i has just left) and so are the block ids of group i+2 ---------------------------
    int blk0, blk1;
    fetch_ids(pair, pos, seg_begin, ctx, blk0, blk1);
    load_group(pair, blk0, blk1);
    load_q(pair);
    reset();
    // position and ids of the next group
    int n_pos = pos + kGroup, n_pair = pair, n_begin = seg_begin, n_end = seg_end, n_ctx = ctx;
    bool n_valid_grp = n_pos < end;
    if (n_valid_grp) {
        while (n_pos >= n_end) seg_of(++n_pair, n_begin, n_end, n_ctx);
        fetch_ids(n_pair, n_pos, n_begin, n_ctx, blk0, blk1);
    }
    while (true) {
        // group (pair, pos) has arrived in f: park it in LDS, then reuse f for the next group
        if constexpr (kFp8) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    u32x4 lo, hi;
                    widen_fp8(f.k[2 * b + j], lo, hi);
                    const int ka = (kw8 ^ (64 * ((2 * j) ^ b))) + 4096 * b + 2048 * j;
                    *reinterpret_cast<u32x4*>(my + ka) = lo;
                    *reinterpret_cast<u32x4*>(my + (ka ^ 16)) = hi;
                    widen_fp8(f.v[2 * b + j], lo, hi);
                    const int va = vw8 + 4096 * b + 2048 * j;
                    *reinterpret_cast<u32x4*>(my + va) = lo;
                    *reinterpret_cast<u32x4*>(my + (va ^ 16)) = hi;
                }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                *reinterpret_cast<u32x4*>(my + kw[j] + 1024 * j) = f.k[j];
                *reinterpret_cast<u32x4*>(my + kw[j ^ 1] + 4096 + 1024 * j) = f.k[4 + j];
                *reinterpret_cast<u32x4*>(my + vw + 1024 * j) = f.v[j];
                *reinterpret_cast<u32x4*>(my + vw + 4096 + 1024 * j) = f.v[4 + j];
            }
        }
        if constexpr (kAppend) {
            const int off_g = pos - seg_begin;
            if (off_g + kGroup >= ctx) {  // uniform: this group holds the pair's last token, position ctx - 1
                const int s_a = pair / hkv_l, g_a = pair % hkv_l;
                const int64_t slot = ap.slots[s_a];
                if (slot >= 0) {
                    const int tl = ctx - 1 - off_g, b = tl >> 4, t = tl & 15;  // block of the group, offset in it
                    const int64_t blk_a = slot / kBlockSize;
                    const int off_a = static_cast<int>(slot % kBlockSize);
                    const size_t row = static_cast<size_t>(s_a) * ap.kv_stride + static_cast<size_t>(g_a) * kD;
                    unsigned char* cache8 = reinterpret_cast<unsigned char*>(cache);
                    if (lane < 16) {  // K row: sixteen 16-byte pieces
                        u32x4 kv = *reinterpret_cast<const u32x4*>(ap.k_new + row + 8 * lane);
                        if constexpr (kFp8) {
                            float x[8];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                x[2 * e] = __uint_as_float(kv[e] << 16);
                                x[2 * e + 1] = __uint_as_float(kv[e] & 0xFFFF0000u);
                            }
                            typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
                            u32x2_t codes;
                            codes[0] = e4m3_pair(x[0], x[1], ap.k_scale) | (e4m3_pair(x[2], x[3], ap.k_scale) << 16);
                            codes[1] = e4m3_pair(x[4], x[5], ap.k_scale) | (e4m3_pair(x[6], x[7], ap.k_scale) << 16);
                            *reinterpret_cast<u32x2_t*>(cache8 + cache_part_offset(blk_a, g_a, 0, hkv_l, kD) + off_a * kD + 8 * lane) = codes;
                            u32x4 lo, hi;
                            widen_fp8(u32x4{codes[0], codes[1], 0u, 0u}, lo, hi);
                            kv = lo;  // what the codes stand for
                        } else {
                            *reinterpret_cast<u32x4*>(cache + cache_part_offset(blk_a, g_a, 0, hkv_l, kD) + off_a * kD + 8 * lane) = kv;
                        }
                        *reinterpret_cast<u32x4*>(my + b * 4096 + t * 256 + ((lane ^ (t & 3) ^ (4 * ((t >> 2) ^ b))) << 4)) = kv;
                    }
#pragma unroll
                    for (int x2 = 0; x2 < 2; ++x2) {  // V column: one element per head-dim row
                        const int d = lane + 64 * x2;
                        uint16_t vv = ap.v_new[row + d];
                        if constexpr (kFp8) {
                            const uint32_t code = e4m3_pair(__uint_as_float(static_cast<uint32_t>(vv) << 16), 0.f, ap.v_scale) & 0xFFu;
                            cache8[cache_part_offset(blk_a, g_a, 1, hkv_l, kD) + static_cast<size_t>(d) * kBlockSize + off_a] =
                                static_cast<unsigned char>(code);
                            typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                            vv = static_cast<uint16_t>(__builtin_bit_cast(
                                uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(code), 1.0f, false)) & 0xFFFFu);
                        } else {
                            cache[cache_part_offset(blk_a, g_a, 1, hkv_l, kD) + static_cast<size_t>(d) * kBlockSize + off_a] = vv;
                        }
                        const int pc = 2 * (d & 31) + (t >> 3);
                        *reinterpret_cast<uint16_t*>(my + 8192 + 4096 * b + 1024 * (d >> 5) + ((pc ^ ((pc >> 4) & 1)) << 4) + 2 * (t & 7)) = vv;
                    }
                }
            }
        }
        int nn_pos = n_pos + kGroup, nn_pair = n_pair, nn_begin = n_begin, nn_end = n_end, nn_ctx = n_ctx;
        bool nn_valid = false;
        if (n_valid_grp) {
            load_group(n_pair, blk0, blk1);
            nn_valid = nn_pos < end;
            if (nn_valid) {
                while (nn_pos >= nn_end) seg_of(++nn_pair, nn_begin, nn_end, nn_ctx);
                fetch_ids(nn_pair, nn_pos, nn_begin, nn_ctx, blk0, blk1);
            }
        }

        f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const bf16x8 ka = as_bf16x8(*reinterpret_cast<const u32x4*>(my + kr[kk]));
            const bf16x8 kb = as_bf16x8(*reinterpret_cast<const u32x4*>(my + kr[kk ^ 1] + 1024));
            sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qf[kk], sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb, qf[kk], sb, 0, 0, 0);
        }
        u32x4 vf[8];
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) vf[mt] = *reinterpret_cast<const u32x4*>(my + vr + 512 * mt);

        const int off = pos - seg_begin;
        const int n_valid = ctx - (off + 8 * grp);
        if (off + kGroup > ctx) {  // last, partial group of the context: uniform branch
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (r >= n_valid) sa[r] = -INFINITY;
                if (4 + r >= n_valid) sb[r] = -INFINITY;
            }
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t mask = n_valid > 2 * w + 1 ? 0xFFFFFFFFu : (n_valid > 2 * w ? 0x0000FFFFu : 0u);
#pragma unroll
                for (int mt = 0; mt < 8; ++mt) vf[mt][w] &= mask;
            }
        }
        float mx = fmaxf(fmaxf(fmaxf(sa[0], sa[1]), fmaxf(sa[2], sa[3])), fmaxf(fmaxf(sb[0], sb[1]), fmaxf(sb[2], sb[3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
        const float mc = m_new * c;
        float pa[4], pb[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            pa[r] = __builtin_amdgcn_exp2f(fmaf(sa[r], c, -mc));
            pb[r] = __builtin_amdgcn_exp2f(fmaf(sb[r], c, -mc));
        }
        l_run = l_run * alpha + ((pa[0] + pa[1]) + (pa[2] + pa[3])) + ((pb[0] + pb[1]) + (pb[2] + pb[3]));
        m_run = m_new;
        bf16x8 pf;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            pf[r] = static_cast<__bf16>(pa[r]);
            pf[4 + r] = static_cast<__bf16>(pb[r]);
        }
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) {
            o[mt] *= alpha;
            o[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vf[mt]), pf, o[mt], 0, 0, 0);
        }
        if (!n_valid_grp) break;
        if (n_pair != pair) {  // the next group starts another pair: emit this one's partial, fetch its queries
            flush(pair);
            reset();
            load_q(n_pair);
        }
        pos = n_pos, pair = n_pair, seg_begin = n_begin, seg_end = n_end, ctx = n_ctx;
        n_pos = nn_pos, n_pair = nn_pair, n_begin = nn_begin, n_end = nn_end, n_ctx = nn_ctx;
        n_valid_grp = nn_valid;
    }
    flush(pair);
}

}  // namespace

namespace {

inline int padded_len(int max_seq_len) { return max_seq_len / kGroup * kGroup + kGroup; }  // >= the padded longest context
// sequences per launch: as many as give the kernel's pair index its fill, and few enough that the padded token line of a
// launch (pairs x padded longest context) stays below 2^31, the range of the kernel's 32-bit prefix sums
inline int seqs_per_launch(int max_seq_len, const AttnShape& a) {
    const int64_t by_line = (static_cast<int64_t>(0x7FFFFFFF) - kGroup) / padded_len(max_seq_len > 0 ? max_seq_len : 1) / a.hkv_l;
    const int64_t by_index = kFlatMaxPairs / a.hkv_l;
    return static_cast<int>(by_line < by_index ? by_line : by_index);
}
// partial rows of a launch over n sequences: one per (wavefront, pair) whose ranges meet, numbered wavefront + pair
inline size_t flat_rows(int n, const AttnShape& a) {
    return (static_cast<size_t>(kFlatWorkers) + static_cast<size_t>(n) * a.hkv_l) * (a.hq_l / a.hkv_l);
}

}  // namespace

bool decode_mfma_supported(const AttnShape& a, int /*num_seqs*/, int max_seq_len) {
    return a.elem == 2 && a.D == kD && a.hq_l % a.hkv_l == 0 && a.hq_l / a.hkv_l <= 16 && a.hkv_l <= kFlatMaxPairs &&
           max_seq_len <= 0x7FFFFFFF - 2 * kGroup && seqs_per_launch(max_seq_len, a) >= 1;
}

size_t decode_mfma_workspace(int num_seqs, int max_seq_len, const AttnShape& a) {
    const int per = seqs_per_launch(max_seq_len, a);
    const int n = num_seqs < per ? num_seqs : per;
    return flat_rows(n, a) * (kD + 2) * sizeof(float) + static_cast<size_t>(n) * a.hkv_l * sizeof(int2);
}

bool decode_mfma_appends(int /*num_seqs*/, const AttnShape& /*a*/) { return true; }

hipError_t launch_decode_mfma(const void* q, const void* k_new, const void* v_new, const int64_t* slots, void* cache,
                              const int32_t* block_table, const int32_t* seq_lens, int num_seqs, int max_seq_len,
                              void* out, void* workspace, const AttnShape& a, hipStream_t st) {
    if (num_seqs == 0) return hipSuccess;  // max_seq_len 0: every row is padding, the kernels write their zeros
    const float c = a.scale * a.k_scale * 1.4426950408889634f;  // logits of an FP8 cache carry k_scale
    // tokens per wavefront never fall below this, so that no output row has more parts than the
    // merge kernel holds (and tiny batches are not shredded into one-group partials)
    const int padded_max = (max_seq_len + kGroup - 1) / kGroup * kGroup;
    int r_min = (padded_max / (kMaxParts - 24) + kGroup) / kGroup * kGroup;
    if (r_min < 2 * kGroup) r_min = 2 * kGroup;
    const bool append = k_new != nullptr;
    const int per = seqs_per_launch(max_seq_len, a);
    for (int s0 = 0; s0 < num_seqs; s0 += per) {  // runs share the workspace: same stream, one after the other
        const int n = num_seqs - s0 < per ? num_seqs - s0 : per;
        const size_t rows = flat_rows(n, a);
        float* o_part = static_cast<float*>(workspace);
        float* ml_part = o_part + rows * kD;
        int2* plan = reinterpret_cast<int2*>(ml_part + rows * 2);
        const uint16_t* q_run = static_cast<const uint16_t*>(q) + static_cast<size_t>(s0) * a.q_stride;
        uint16_t* out_run = static_cast<uint16_t*>(out) + static_cast<size_t>(s0) * a.out_stride;
        const AppendArgs ap = {append ? static_cast<const uint16_t*>(k_new) + static_cast<size_t>(s0) * a.kv_stride : nullptr,
                               append ? static_cast<const uint16_t*>(v_new) + static_cast<size_t>(s0) * a.kv_stride : nullptr,
                               append ? slots + s0 : nullptr, a.kv_stride, a.k_scale, a.v_scale};
        auto launch = [&](auto kernel) {
            kernel<<<kFlatWorkgroups, kWaves * 64, 0, st>>>(q_run, a.q_stride, static_cast<uint16_t*>(cache),
                                                            block_table + static_cast<size_t>(s0) * a.max_blocks, a.max_blocks,
                                                            seq_lens + s0, o_part, ml_part, plan, n, a.hq_l, a.hkv_l, c, r_min, ap);
        };
        if (a.kv_fp8()) {
            if (append) launch(decode_flat_kernel<true, true>);
            else launch(decode_flat_kernel<true, false>);
        } else {
            if (append) launch(decode_flat_kernel<false, true>);
            else launch(decode_flat_kernel<false, false>);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        e = launch_combine_flat(o_part, ml_part, plan, n, a.hq_l, a.hq_l / a.hkv_l, out_run, a.out_stride, a.v_scale, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace shiftattn
