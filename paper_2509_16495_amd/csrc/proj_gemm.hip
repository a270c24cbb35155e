// The two projections that touch the exchange (Algorithm 1: qkv = embed * W_qkv in front of the first
// all-to-all, embed = attn_o * W_o behind the second), as one bf16 MFMA GEMM whose operand and result
// addressing carries the pack / unpack:
//   qkv_proj_pack : C[t][f] = sum_k x[t][k] W[f][k]; feature tile f lies in one head, and a head's
//                   columns go straight to the send buffer(s) of the rank(s) that own it (Sec. 3.2.1:
//                   fused q|k|v exchange, KV replication) - the pack kernel and its round trip
//                   through HBM disappear;
//   unpack_o_proj : C[t][c] = sum_k a[t][k] W_o[c][k] with a[t][(p hq_l + j) D + e] read in place from
//                   receive buffer p - the unpack kernel disappears.
// Weights are stored one row per output feature (K contiguous), as linear layers keep them.
//
// Kernel: 256 x 256 output tile per workgroup, K in tiles of 32, four wavefronts (2 along the features
// x 2 along the tokens, 128 x 128 each: one wavefront per SIMD with its 256 accumulator registers in the
// AGPR half of the register file), v_mfma_f32_32x32x16_bf16 with the weight rows as A operand and the
// token rows as B operand, so a lane ends up with runs of four consecutive features of one token (8-byte
// stores).  The two operand tiles of a k tile (2 x 16 KiB) arrive by direct-to-LDS loads into a ring of
// four buffers: one is multiplied while up to three are in flight, and the wait in front of the one
// meeting per k tile counts loads instead of draining them.  A row of 32 k (64 bytes) keeps its four
// 16-byte pieces at positions piece ^ ((row / 4) % 4), which makes the operand reads (32 consecutive
// rows, one piece column) conflict-free.
#include "internal.h"

#include <type_traits>

namespace shiftattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int kTile = 256;                 // rows of either operand per workgroup
constexpr int kRowBytes = 64;              // bytes of a row per k tile: 32 bf16 or 64 FP8 elements
constexpr int kOperandBytes = kTile * kRowBytes;   // 16384
constexpr int kStage = 2 * kOperandBytes;  // weights, then tokens
constexpr int kStages = 4;                 // ring of k tiles in LDS: one being multiplied, the others in flight
constexpr int kGemmLds = kStages * kStage; // 131072
constexpr int kWavesN = 2, kWavesM = 2;    // wavefronts along the features / along the tokens
constexpr int kGemmThreads = 64 * kWavesN * kWavesM;
constexpr int kNT = kTile / kWavesN / 32;  // 32-feature tiles per wavefront
constexpr int kMT = kTile / kWavesM / 32;  // 32-token tiles per wavefront
constexpr int kLoadRows = kTile / (kWavesN * kWavesM);   // rows of either operand that one wavefront loads
constexpr int kLoadsPerOperand = kLoadRows / 16;          // 16 rows (1 KiB) per instruction
constexpr int kLoadsPerTile = 2 * kLoadsPerOperand;       // direct-to-LDS instructions per wavefront and k tile
constexpr int kLoadEvery = kNT * kMT / kLoadsPerOperand;  // MFMAs between two loads
static_assert(kNT * kMT % kLoadsPerOperand == 0 && kNT + kMT <= 15, "load spreading / lgkmcnt field");

// s_waitcnt immediates: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8
constexpr int wait_imm(int vm, int lgkm) { return (vm & 15) | ((vm >> 4) << 14) | 0x70 | (lgkm << 8); }
constexpr int kNoVm = 63, kNoLgkm = 15;
constexpr int kHeadDim = 128;

__device__ inline bf16x8 frag(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct GemmParams {
    const unsigned char* __restrict__ w;   // [N][K], bf16 or FP8 E4M3 codes
    const unsigned char* __restrict__ x;   // token rows of the same type; see mode
    uint16_t* __restrict__ c;              // bf16
    const float* __restrict__ xs;          // FP8: one scale per token row
    const float* __restrict__ ws;          // FP8: one scale per output feature
    int M, M_out, N, K;               // M token rows exist, rows M..M_out-1 of the result are written as zeros
    // mode 0 (qkv_proj_pack): x dense [M][K]; result columns scattered to send buffers (XchgShape below)
    // mode 1 (unpack_o_proj): x gathered from recv [P][T_pad][hq_l][128] (k = (p hq_l + j) 128 + e); result dense [M][N]
    int mode;
    int k_splits;                     // workgroups that share an output tile, each with a range of k tiles (bf16 only)
    float* __restrict__ partial;      // k_splits > 1: fp32 partial results [k_splits][M_out][N] instead of c
    XchgShape s;
};

// kFp8: both operands are FP8 E4M3 codes (v_mfma_scale_f32_32x32x64_f8f6f4 with unit block scales, fp32
// accumulation); the result is multiplied by the token's and the feature's scale before it is rounded to bf16.
// kSplit: the workgroup covers one of p.k_splits ranges of k and leaves fp32 sums in p.partial (for FP8 operands: before
// the scales, which the finishing kernel applies)
template <bool kFp8, bool kSplit>
__global__ __launch_bounds__(kGemmThreads) void proj_gemm_kernel(GemmParams p) {
    constexpr int kElem = kFp8 ? 1 : 2;          // bytes per operand element
    constexpr int kBK = kRowBytes / kElem;       // k per tile
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    typedef __attribute__((address_space(3))) void* lds_ptr;
    typedef const __attribute__((address_space(1))) void* glb_ptr;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, half = lane >> 5;
    const int wn = wave % kWavesN, wm = wave / kWavesN;
    // feature tiles vary fastest: workgroups that run together share the token rows in L2
    const int n_tiles = p.N / kTile;
    const int n_splits = kSplit ? p.k_splits : 1;
    const int tile_id = blockIdx.x / n_splits, split = blockIdx.x - tile_id * n_splits;
    const int n0 = (tile_id % n_tiles) * kTile, m0 = (tile_id / n_tiles) * kTile;
    // this workgroup's k tiles: [kt0, kt0 + k_steps) of the K / kBK in all
    const int kt_all = p.K / kBK;
    const int kt0 = kSplit ? static_cast<int>(static_cast<int64_t>(kt_all) * split / n_splits) : 0;
    const int k_steps = kSplit ? static_cast<int>(static_cast<int64_t>(kt_all) * (split + 1) / n_splits) - kt0 : kt_all;

    // ---- direct-to-LDS loads: this wavefront fills rows 32 wave .. 32 wave + 31 of both operand tiles, sixteen rows
    // (1 KiB) per instruction; lane -> row 16 j + lane / 4, LDS piece position lane % 4, logical piece = position ^ key
    // The address of a load is a wavefront-uniform base (tile origin + k, kept in scalar registers and advanced by
    // scalar adds) plus a 32-bit byte offset per lane that never changes, and the LDS destination is uniform too: no
    // vector ALU instruction is spent on a load.
    const int ld_row = lane >> 2, ld_pos = lane & 3;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const size_t k_bytes = static_cast<size_t>(p.K) * kElem;
    const size_t seg_bytes = p.mode == 0 ? k_bytes : static_cast<size_t>(p.s.hq_l) * kHeadDim * kElem;   // contiguous k of a token row
    uint32_t w_off[kLoadsPerOperand], x_off[kLoadsPerOperand];   // byte offsets of this lane's piece from the tile origin at k = 0
#pragma unroll
    for (int j = 0; j < kLoadsPerOperand; ++j) {
        const int row = kLoadRows * wave + 16 * j + ld_row;
        const int piece = ld_pos ^ ((row >> 2) & 3);
        w_off[j] = static_cast<uint32_t>(static_cast<size_t>(row) * k_bytes + piece * 16);
        const int m = min(m0 + row, p.M - 1) - m0;   // rows past the end re-read the last one; they are not stored
        x_off[j] = static_cast<uint32_t>(static_cast<size_t>(m) * seg_bytes + piece * 16);
    }
    const unsigned char* w_tile = p.w + static_cast<size_t>(n0) * k_bytes;
    const unsigned char* x_tile = p.x + static_cast<size_t>(m0) * seg_bytes;
    // A token row's k runs contiguously through the hq_l heads that one source rank returned, then jumps to the
    // next rank's buffer (mode 1); in mode 0 it is contiguous throughout.
    const int seg_tiles = static_cast<int>(seg_bytes / kRowBytes);
    const size_t seg_jump = p.mode == 0 ? 0 : static_cast<size_t>(p.s.T_pad - 1) * seg_bytes;
    int ld_kt = 0, ld_left = seg_tiles - kt0 % seg_tiles;   // next tile to load (counted from kt0), and how many tiles remain in its segment
    w_tile += static_cast<size_t>(kt0) * kRowBytes;
    x_tile += static_cast<size_t>(kt0) * kRowBytes + static_cast<size_t>(kt0 / seg_tiles) * seg_jump;
    // 1 KiB from a wavefront-uniform base (scalar registers) + a 32-bit byte offset per lane into LDS at dst (uniform):
    // written as assembly so that the load forms the address itself instead of a 64-bit vector addition in front of it.
    // These loads are waited for with the explicit vmcnt waits below only.
    auto scalar_ptr = [](const unsigned char* ptr) -> const unsigned char* {
        const uint64_t a = reinterpret_cast<uint64_t>(ptr);
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
        return reinterpret_cast<const unsigned char*>((static_cast<uint64_t>(hi) << 32) | lo);
    };
    auto dma_1k = [&](const unsigned char* base, uint32_t lane_off, unsigned char* dst) {
        const uint32_t m0v = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(dst));
        // (M0 is reserved by the compiler - it sets it right before each use of its own and keeps no value in it, and
        // rejects it on a clobber list - so writing it here needs no clobber.)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(m0v), "v"(lane_off), "s"(scalar_ptr(base)) : "memory");
    };
    auto load_one = [&](int j) {          // first the weight rows, then the token rows
        unsigned char* dst = lds + (ld_kt % kStages) * kStage + (kLoadRows * wave_s) * kRowBytes;
        if (j < kLoadsPerOperand) dma_1k(w_tile, w_off[j], dst + j * 1024);
        else dma_1k(x_tile, x_off[j - kLoadsPerOperand], dst + kOperandBytes + (j - kLoadsPerOperand) * 1024);
    };
    auto load_advance = [&]() {
        ++ld_kt;
        w_tile += kRowBytes;
        x_tile += kRowBytes;
        if (--ld_left == 0) { ld_left = seg_tiles; x_tile += seg_jump; }
    };

    // ---- operand reads: row l32 of a 32-row tile, piece 2 ks + half
    const int key = (l32 >> 2) & 3;   // 32-row tiles start at multiples of 32: the key depends on l32 only
    int rd[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) rd[ks] = l32 * kRowBytes + (((2 * ks + half) ^ key) << 4);
    const int a_base = (wn * kNT * 32) * kRowBytes;                    // weight rows of this wavefront
    const int b_base = kOperandBytes + (wm * kMT * 32) * kRowBytes;   // token rows of this wavefront

    f32x16 acc[kNT][kMT];
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
        for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nt][mt][r] = 0.f;

    // Operands are read from LDS one 16-wide k slice ahead of the MFMAs that use them (two register sets).  The
    // workgroup meets once per k tile, before the tile's last slice is multiplied: by then every wavefront holds
    // that slice in registers, so the tile's buffer is free, and the first slice of the next tile is fetched while
    // the last one is multiplied.  The loads of the tile kStages - 1 ahead go into the buffer freed one meeting
    // earlier and are spread between the MFMAs, one behind every fourth.
    auto read_ops = [&](const unsigned char* base, int ks, u32x4 (&a)[kNT], u32x4 (&b)[kMT]) {
#pragma unroll
        for (int nt = 0; nt < kNT; ++nt) a[nt] = *reinterpret_cast<const u32x4*>(base + a_base + nt * 32 * kRowBytes + rd[ks]);
#pragma unroll
        for (int mt = 0; mt < kMT; ++mt) b[mt] = *reinterpret_cast<const u32x4*>(base + b_base + mt * 32 * kRowBytes + rd[ks]);
    };
    auto multiply = [&]<int kLoad0>(const u32x4 (&a)[kNT], const u32x4 (&b)[kMT]) {   // kLoad0 < 0: no loads in between
#pragma unroll
        for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt) {
                acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[nt]), frag(b[mt]), acc[nt][mt], 0, 0, 0);
                if (kLoad0 >= 0 && (nt * kMT + mt) % kLoadEvery == 1) {
                    load_one(kLoad0 + (nt * kMT + mt) / kLoadEvery);
                    __builtin_amdgcn_sched_barrier(0);   // keep the load between these MFMAs
                }
            }
    };

    auto prologue = [&]() {   // the first kStages - 1 tiles are requested, tile 0 has landed everywhere
        for (int t = 0; t < kStages - 1 && t < k_steps; ++t) {
#pragma unroll
            for (int j = 0; j < kLoadsPerTile; ++j) load_one(j);
            load_advance();
        }
        if (k_steps >= kStages - 1) __builtin_amdgcn_s_waitcnt(wait_imm(kLoadsPerTile * (kStages - 2), kNoLgkm));
        else __builtin_amdgcn_s_waitcnt(wait_imm(0, kNoLgkm));
        __builtin_amdgcn_s_barrier();
    };
    if constexpr (!kFp8) {
        u32x4 a0[kNT], b0[kMT], a1[kNT], b1[kMT];
        prologue();
        read_ops(lds, 0, a0, b0);
        auto tile = [&]<bool kLoads>(int kt) {
            read_ops(lds + (kt % kStages) * kStage, 1, a1, b1);
            __builtin_amdgcn_sched_barrier(0);   // the reads stay ahead of the MFMAs of the slice before ...
            __builtin_amdgcn_s_waitcnt(wait_imm(kNoVm, kNT + kMT));  // ... which wait for their own operands only
            multiply.template operator()<kLoads ? 0 : -1>(a0, b0);
            // tile kt + 1 has landed (behind it: kStages - 3 whole tiles and the weight loads just issued), and this
            // wavefront's reads of tile kt are done
            __builtin_amdgcn_sched_barrier(0);
            if (kLoads) __builtin_amdgcn_s_waitcnt(wait_imm(kLoadsPerTile * (kStages - 3) + kLoadsPerOperand, 0));
            else __builtin_amdgcn_s_waitcnt(wait_imm(0, 0));
            __builtin_amdgcn_s_barrier();   // bare: a __syncthreads() would wait for every load in flight
            read_ops(lds + ((kt + 1) % kStages) * kStage, 0, a0, b0);   // behind the last tile: stale data, not used
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_waitcnt(wait_imm(kNoVm, kNT + kMT));
            multiply.template operator()<kLoads ? kLoadsPerOperand : -1>(a1, b1);
            if (kLoads) load_advance();
        };
        int kt = 0;
        for (; kt + kStages - 1 < k_steps; ++kt) tile.template operator()<true>(kt);
        for (; kt < k_steps; ++kt) tile.template operator()<false>(kt);
    } else {
        // One MFMA per (feature tile, token tile) and k tile: its 32-byte operands are the two 16-byte pieces the
        // bf16 path reads for its two k slices (which k a lane holds does not matter as long as both operands agree).
        // Two register sets: the next tile's operands are fetched while this tile's MFMAs run.
        i32x8 a[2][kNT], b[2][kMT];   // [set]
        auto join = [](u32x4 lo, u32x4 hi) -> i32x8 {
            return i32x8{static_cast<int>(lo[0]), static_cast<int>(lo[1]), static_cast<int>(lo[2]), static_cast<int>(lo[3]),
                         static_cast<int>(hi[0]), static_cast<int>(hi[1]), static_cast<int>(hi[2]), static_cast<int>(hi[3])};
        };
        auto read_tile = [&](const unsigned char* base, auto set_c) {
            constexpr int S = decltype(set_c)::value;
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt) {
                const unsigned char* r = base + a_base + nt * 32 * kRowBytes;
                a[S][nt] = join(*reinterpret_cast<const u32x4*>(r + rd[0]), *reinterpret_cast<const u32x4*>(r + rd[1]));
            }
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt) {
                const unsigned char* r = base + b_base + mt * 32 * kRowBytes;
                b[S][mt] = join(*reinterpret_cast<const u32x4*>(r + rd[0]), *reinterpret_cast<const u32x4*>(r + rd[1]));
            }
        };
        // kLoadMode 1: the tile kStages - 1 ahead exists and is requested; 2: checked at run time (the last few tiles)
        auto tile8 = [&]<int kLoadMode, int S>(int kt) {
            const bool ld = kLoadMode == 1 || kt + kStages - 1 < k_steps;
            // tile kt + 1 has landed (behind it kStages - 3 whole tiles), and this wavefront's reads of tile kt are done
            if (ld) __builtin_amdgcn_s_waitcnt(wait_imm(kLoadsPerTile * (kStages - 3), 0));
            else __builtin_amdgcn_s_waitcnt(wait_imm(0, 0));
            __builtin_amdgcn_s_barrier();
            read_tile(lds + ((kt + 1) % kStages) * kStage, std::integral_constant<int, 1 - S>{});   // behind the last tile: stale, unused
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
                for (int mt = 0; mt < kMT; ++mt) {
                    acc[nt][mt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[S][nt], b[S][mt], acc[nt][mt], 0, 0, 0, 127, 0, 127);
                    if ((nt * kMT + mt) % 2 == 0) {
                        if (ld) load_one((nt * kMT + mt) / 2);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            if (ld) load_advance();
        };
        static_assert(kNT * kMT == 2 * kLoadsPerTile, "one load behind every second MFMA");
        prologue();
        read_tile(lds, std::integral_constant<int, 0>{});
        int kt = 0;
        for (; kt + kStages < k_steps; kt += 2) {
            tile8.template operator()<1, 0>(kt);
            tile8.template operator()<1, 1>(kt + 1);
        }
        for (; kt < k_steps; kt += 2) {
            tile8.template operator()<2, 0>(kt);
            if (kt + 1 < k_steps) tile8.template operator()<2, 1>(kt + 1);
        }
    }

    // ---- result: register r of acc[nt][mt] is feature 32 nt + 8 (r / 4) + 4 half + r % 4 of token 32 mt + l32
    const int f_wave = n0 + wn * kNT * 32;     // first feature of this wavefront; its features lie in one head
    auto store_rows = [&](uint16_t* dst_row0, size_t row_stride) {   // dst_row0: feature f_wave of token row 0
#pragma unroll
        for (int mt = 0; mt < kMT; ++mt) {
            const int m = m0 + wm * kMT * 32 + mt * 32 + l32;
            if (m >= p.M_out) continue;
            uint16_t* row = dst_row0 + static_cast<size_t>(m) * row_stride + 4 * half;
            float row_scale = 1.f;
            if constexpr (kFp8) row_scale = m < p.M ? p.xs[m] : 0.f;
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    f32x4 col_scale = {1.f, 1.f, 1.f, 1.f};
                    if constexpr (kFp8) col_scale = *reinterpret_cast<const f32x4*>(p.ws + f_wave + 32 * nt + 8 * r4 + 4 * half);
                    bf16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float y = m < p.M ? acc[nt][mt][4 * r4 + e] : 0.f;
                        if constexpr (kFp8) y = y * row_scale * col_scale[e];
                        v[e] = static_cast<__bf16>(y);
                    }
                    *reinterpret_cast<u32x2*>(row + 32 * nt + 8 * r4) = __builtin_bit_cast(u32x2, v);
                }
        }
    };
    if constexpr (kSplit) {   // this k range's fp32 sums, [split][token][feature]; proj_finish adds the ranges and does the layout
        float* base = p.partial + static_cast<size_t>(split) * p.M_out * p.N + f_wave + 4 * half;
#pragma unroll
        for (int mt = 0; mt < kMT; ++mt) {
            const int m = m0 + wm * kMT * 32 + mt * 32 + l32;
            if (m >= p.M) continue;   // rows past the last token are zeros in the result and are not read
            float* row = base + static_cast<size_t>(m) * p.N;
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4)
                    *reinterpret_cast<f32x4*>(row + 32 * nt + 8 * r4) =
                        f32x4{acc[nt][mt][4 * r4], acc[nt][mt][4 * r4 + 1], acc[nt][mt][4 * r4 + 2], acc[nt][mt][4 * r4 + 3]};
        }
        return;
    }
    if (p.mode == 1) {
        store_rows(p.c + f_wave, static_cast<size_t>(p.N));
        return;
    }
    // send buffers [P][T_pad][hq_l + 2 hkv_l][128]: which buffer(s) own this head (wavefront-uniform)
    const XchgShape& s = p.s;
    const int head = f_wave / kHeadDim, col = f_wave % kHeadDim;
    const int w_out = s.hq_l + 2 * s.hkv_l;
    const size_t row_stride = static_cast<size_t>(w_out) * kHeadDim;
    const size_t buf_stride = static_cast<size_t>(s.T_pad) * row_stride;
    if (head < s.h) {
        const int dest = head / s.hq_l, local = head - dest * s.hq_l;
        store_rows(p.c + dest * buf_stride + local * kHeadDim + col, row_stride);
    } else {
        const bool is_v = head >= s.h + s.h_kv;
        const int g = head - s.h - (is_v ? s.h_kv : 0);   // K or V head on the source side
        const int slot0 = s.hq_l + (is_v ? s.hkv_l : 0);
        if (s.h_kv >= s.P) {   // each destination owns hkv_l consecutive heads
            const int dest = g / s.hkv_l, local = slot0 + (g - dest * s.hkv_l);
            store_rows(p.c + dest * buf_stride + local * kHeadDim + col, row_stride);
        } else {               // replication: head g goes to the P / h_kv destinations whose first KV head it is
            for (int dest = 0; dest < s.P; ++dest)
                if (static_cast<int>((static_cast<int64_t>(dest) * s.h_kv) / s.P) == g)
                    store_rows(p.c + dest * buf_stride + slot0 * kHeadDim + col, row_stride);
        }
    }
}

template <bool kFp8>
hipError_t launch(const GemmParams& p, hipStream_t st) {
    const int64_t wgs = static_cast<int64_t>(p.N / kTile) * ((p.M_out + kTile - 1) / kTile) * p.k_splits;
    if (wgs == 0) return hipSuccess;
    if (wgs > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (p.k_splits > 1) {
        proj_gemm_kernel<kFp8, true><<<static_cast<unsigned>(wgs), kGemmThreads, kGemmLds, st>>>(p);
        return hipGetLastError();
    }
    proj_gemm_kernel<kFp8, false><<<static_cast<unsigned>(wgs), kGemmThreads, kGemmLds, st>>>(p);
    return hipGetLastError();
}

// Few output tiles (up to about a thousand token rows): k is split over workgroups when a rough model of the launch
// says so - a workgroup walks its k range at about 6.5 TFLOP/s (12.5 over FP8 operands), workgroups beyond one per compute unit queue up in
// rounds, and every range adds fp32 partial results that are written and read back.  Ranges are at least 16 k tiles
// long.  1: no split (enough tiles or a short k).
int k_splits_for(int M_out, int N, int K, bool fp8) {
    const int64_t tiles = static_cast<int64_t>(N / kTile) * ((M_out + kTile - 1) / kTile);
    if (tiles == 0 || tiles >= 512) return 1;
    const double walk = 2.0 * kTile * kTile * static_cast<double>(K) / (fp8 ? 12.5e12 : 6.5e12);   // one workgroup over all of k
    const double partial = 2.0 * M_out * static_cast<double>(N) * sizeof(float) / 4.0e12;
    auto model = [&](int sp) {
        const double load = static_cast<double>(tiles) * sp / 256.0;
        const double whole = static_cast<double>(static_cast<long>(load + 0.999999));
        const double rounds = load <= 1.0 ? 1.0 : (whole < load + 0.5 ? whole : load + 0.5);
        return rounds / sp * walk + (sp > 1 ? sp * partial + 5.0e-6 : 0.0);
    };
    const int by_length = K / (fp8 ? 64 : 32) / 16;
    int best = 1;
    double t_best = model(1);
    for (int sp = 2; sp <= 16 && sp <= by_length; ++sp) {
        const double t = model(sp);
        if (t < 0.97 * t_best) {
            t_best = t;
            best = sp;
        }
    }
    return best;
}

}  // namespace

// bf16, head_dim 128; the feature dimension of either product must be a multiple of the 256-wide tile
hipError_t proj_gemm_init() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&proj_gemm_kernel<false, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&proj_gemm_kernel<false, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&proj_gemm_kernel<true, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&proj_gemm_kernel<true, true>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
}

bool qkv_proj_pack_supported(const XchgShape& s, int d_model, int elem) {
    return elem == 2 && s.vec_per_head * 8 == kHeadDim && d_model > 0 && d_model % 64 == 0 && (s.h + 2 * s.h_kv) % 2 == 0;
}
bool unpack_o_proj_supported(const XchgShape& s, int d_model, int elem) {
    return elem == 2 && s.vec_per_head * 8 == kHeadDim && d_model > 0 && d_model % kTile == 0 && s.h > 0;
}

size_t proj_gemm_workspace(int M_out, int N, int K, bool fp8) {
    const int sp = k_splits_for(M_out, N, K, fp8);
    return sp == 1 ? 0 : static_cast<size_t>(sp) * M_out * N * sizeof(float);
}

// runs the product with its k split when that pays and the workspace holds the partial results
static hipError_t run_gemm(GemmParams& p, void* workspace, size_t workspace_bytes, hipStream_t st) {
    p.k_splits = 1;
    p.partial = nullptr;
    const bool fp8 = p.xs != nullptr;
    const size_t need = proj_gemm_workspace(p.M_out, p.N, p.K, fp8);
    if (need == 0 || need > workspace_bytes || !workspace) return fp8 ? launch<true>(p, st) : launch<false>(p, st);
    p.k_splits = k_splits_for(p.M_out, p.N, p.K, fp8);
    p.partial = static_cast<float*>(workspace);
    const hipError_t e = fp8 ? launch<true>(p, st) : launch<false>(p, st);
    if (e != hipSuccess) return e;
    return launch_proj_finish(p.partial, p.k_splits, p.M_out, p.c, p.M, p.M_out, p.N, p.mode, p.s, p.xs, p.ws, st);
}

hipError_t launch_qkv_proj_pack(const void* x, const void* w_qkv, void* send, int d_model, const XchgShape& s,
                                const float* x_scales, const float* w_scales, void* workspace, size_t workspace_bytes,
                                hipStream_t st) {
    GemmParams p;
    p.w = static_cast<const unsigned char*>(w_qkv);
    p.x = static_cast<const unsigned char*>(x);
    p.c = static_cast<uint16_t*>(send);
    p.xs = x_scales;
    p.ws = w_scales;
    p.M = s.T;
    p.M_out = s.T_pad;
    p.N = (s.h + 2 * s.h_kv) * kHeadDim;
    p.K = d_model;
    p.mode = 0;
    p.s = s;
    if (s.T == 0) return launch_pack(nullptr, send, s, st);  // only padding rows: the pack kernel writes the zeros
    return run_gemm(p, workspace, workspace_bytes, st);
}

hipError_t launch_unpack_o_proj(const void* recv, const void* w_o, void* out, int d_model, const XchgShape& s,
                                const float* a_scales, const float* w_scales, void* workspace, size_t workspace_bytes,
                                hipStream_t st) {
    GemmParams p;
    p.w = static_cast<const unsigned char*>(w_o);
    p.x = static_cast<const unsigned char*>(recv);
    p.c = static_cast<uint16_t*>(out);
    p.xs = a_scales;
    p.ws = w_scales;
    p.M = s.T;
    p.M_out = s.T;
    p.N = d_model;
    p.K = s.h * kHeadDim;
    p.mode = 1;
    p.s = s;
    if (s.T == 0) return hipSuccess;
    return run_gemm(p, workspace, workspace_bytes, st);
}

}  // namespace shiftattn
