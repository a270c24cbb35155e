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
// Kernel: 256 x 256 output tile per workgroup, four wavefronts (2 along the features x 2 along the tokens, 128 x 128
// each: one wavefront per SIMD with its 256 accumulator registers in the AGPR half of the register file), the weight
// rows as A operand and the token rows as B operand, so a lane ends up with runs of four consecutive features of one
// token (8-byte stores).  k advances in stages of 128 bytes per row (64 bf16 or 128 FP8 elements: whole cache lines),
// two stage buffers of 64 KiB in LDS filled by direct-to-LDS loads of 1 KiB (eight rows); a row keeps its eight
// 16-byte pieces at positions piece ^ ((row / 2) % 8), which makes the operand reads (16 or 32 consecutive rows, one
// piece column) conflict-free.  One barrier per stage.  bf16: v_mfma_f32_16x16x32_bf16; FP8: v_mfma_scale_f32_16x16x128_f8f6f4.
// What the main loop is built around (all measured on this kernel):
//   * the chip runs these kernels at its power limit: the clock settles where MFMA rate x energy per MFMA fits, so
//     the 16x16x32 form (less accumulator traffic per flop) sustains about 15 % more than 32x32x16;
//   * with one wavefront per SIMD and 16-clock MFMAs the matrix pipe stays fed only if at most one other instruction
//     sits between two MFMAs: every LDS read, every load (split in two: M0, then the load) and the scalar bookkeeping
//     has a slot of its own behind an MFMA;
//   * workgroups on different XCDs start their walk over k at different places (see rot0 below).
#include "internal.h"

#include <type_traits>
#include <utility>

namespace shiftattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int kTile = 256;                 // rows of either operand per workgroup
constexpr int kRowBytes = 128;             // bytes of a row per k stage: one cache line, 64 bf16 or 128 FP8 elements
constexpr int kOperandBytes = kTile * kRowBytes;   // 32768
constexpr int kStage = 2 * kOperandBytes;  // weights, then tokens
constexpr int kStages = 2;                 // k stages in LDS: one being multiplied, one in flight
constexpr int kStagingPitch = 272;         // bytes between token rows of a wavefront's result staged in LDS (256 + 16)
constexpr int kStagingWave = (kTile / 2) * kStagingPitch;   // 128 token rows per wavefront
constexpr int kGemmLds = 4 * kStagingWave > kStages * kStage ? 4 * kStagingWave : kStages * kStage;   // 139264
constexpr int kWavesN = 2, kWavesM = 2;    // wavefronts along the features / along the tokens
constexpr int kGemmThreads = 64 * kWavesN * kWavesM;
constexpr int kWaveRows = kTile / kWavesN;                // rows of either operand that one wavefront multiplies (128)
static_assert(kTile / kWavesM == kWaveRows, "square wavefront tiles");
constexpr int kLoadRows = kTile / (kWavesN * kWavesM);   // rows of either operand that one wavefront loads
constexpr int kLoadsPerOperand = kLoadRows / 8;           // 8 rows (1 KiB) per instruction
constexpr int kLoadsPerStage = 2 * kLoadsPerOperand;      // direct-to-LDS instructions per wavefront and k stage

// s_waitcnt immediates: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8
constexpr int wait_imm(int vm, int lgkm) { return (vm & 15) | ((vm >> 4) << 14) | 0x70 | (lgkm << 8); }
constexpr int kNoVm = 63, kNoLgkm = 15;
constexpr int kHeadDim = 128;

__device__ inline bf16x8 frag(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// The bf16 MFMA as assembly with its accumulator tied in place in an accumulation register: given the builtin, the
// register allocator rotated the 64 small accumulators of a wavefront through both register files (some 500 copies
// per k stage).  The compiler does not know this statement is an MFMA: its operands come straight from LDS reads
// (waited for by the compiler, which does track the registers), an accumulator is touched again 64 MFMAs later at the
// earliest, and compiler-generated reads of the results sit behind mfma_settle().
__device__ inline __attribute__((always_inline)) void mfma_16x16x32(f32x4& d, u32x4 a, u32x4 b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}
__device__ inline __attribute__((always_inline)) void mfma_settle() { asm volatile("s_nop 7\n\ts_nop 7" ::: "memory"); }

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
    int k_splits;                     // workgroups that share an output tile, each with a range of k stages
    float* __restrict__ partial;      // k_splits > 1: fp32 partial results [k_splits][M_out - m_base][N] instead of c
    int items;                        // work items of the launch: output tiles x k ranges
    int m_base;                       // first token row of the launch's tiles (a multiple of the tile height)
    int m_tiles;                      // token tiles of the launch
    XchgShape s;
};

// kFp8: both operands are FP8 E4M3 codes (v_mfma_scale_f32_16x16x128_f8f6f4 with unit block scales, fp32
// accumulation); the result is multiplied by the token's and the feature's scale before it is rounded to bf16.
// kSplit: the workgroup covers one of p.k_splits ranges of k and leaves fp32 sums in p.partial (for FP8 operands: before
// the scales, which the finishing kernel applies).  One call is one output tile (and k range): work item `item` of the launch.
template <bool kFp8, bool kSplit>
__device__ __attribute__((always_inline)) void proj_gemm_tile(const GemmParams& p, const int item) {
    constexpr int kElem = kFp8 ? 1 : 2;          // bytes per operand element
    constexpr int kBK = kRowBytes / kElem;       // k per stage
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    // (an opaque copy of the thread index per work item, and another one for the epilogue below: as invariants of the
    // persistent loop, everything derived from it would be computed once and kept in registers through the main loop)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int wave = tid >> 6, lane = tid & 63;
    const int wn = wave % kWavesN, wm = wave / kWavesN;
    // feature tiles vary fastest: workgroups that run together share the token rows in L2
    const int n_tiles = p.N / kTile;
    const int n_splits = kSplit ? p.k_splits : 1;
    const int tile_id = item / n_splits, split = item - tile_id * n_splits;
    const int n0 = (tile_id % n_tiles) * kTile, m0 = p.m_base + (tile_id / n_tiles) * kTile;
    // this workgroup's k stages: [kt0, kt0 + k_steps) of all; with FP8 operands the very last stage may hold 64 k only
    const int kt_all = (p.K + kBK - 1) / kBK;
    const int kt0 = kSplit ? static_cast<int>(static_cast<int64_t>(kt_all) * split / n_splits) : 0;
    const int k_steps = kSplit ? static_cast<int>(static_cast<int64_t>(kt_all) * (split + 1) / n_splits) - kt0 : kt_all;
    const bool ragged = kFp8 && p.K % kBK != 0 && kt0 + k_steps == kt_all;

    // ---- direct-to-LDS loads: this wavefront fills rows 64 wave .. 64 wave + 63 of both operand tiles, eight rows of
    // 128 bytes (1 KiB, eight whole cache lines) per instruction; lane -> row 8 j + lane / 8, LDS piece position
    // lane % 8, logical piece = position ^ key.  (Half lines - 16 rows of 64 bytes per instruction - kept the address
    // path of the compute unit busy nine tenths of the time and every line was requested twice, one k tile apart.)
    // The address of a load is a wavefront-uniform base (tile origin + k, kept in scalar registers and advanced by
    // scalar adds) plus a 32-bit byte offset per lane that never changes, and the LDS destination is uniform too: no
    // vector ALU instruction is spent on a load.
    const int ld_row = lane >> 3, ld_pos = lane & 7;
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const size_t k_bytes = static_cast<size_t>(p.K) * kElem;
    const size_t seg_bytes = p.mode == 0 ? k_bytes : static_cast<size_t>(p.s.hq_l) * kHeadDim * kElem;   // contiguous k of a token row
    uint32_t w_off[kLoadsPerOperand], x_off[kLoadsPerOperand];   // byte offsets of this lane's piece from the tile origin at k = 0
#pragma unroll
    for (int j = 0; j < kLoadsPerOperand; ++j) {
        const int row = kLoadRows * wave + 8 * j + ld_row;
        const int piece = ld_pos ^ ((row >> 1) & 7);
        w_off[j] = static_cast<uint32_t>(static_cast<size_t>(row) * k_bytes + piece * 16);
        const int m = min(m0 + row, p.M - 1) - m0;   // rows past the end re-read the last one; they are not stored
        x_off[j] = static_cast<uint32_t>(static_cast<size_t>(m) * seg_bytes + piece * 16);
    }
    // A half-filled last stage: the lanes of pieces 4..7 (past the end of the row) fetch pieces 0..3 once more.  The
    // key of row 64 wave + 8 j + lane / 8 has bit 2 equal to j % 2, so which lanes those are depends on j % 2 only.
    uint32_t tail_fix[2];
#pragma unroll
    for (int jp = 0; jp < 2; ++jp) tail_fix[jp] = (((ld_pos >> 2) ^ jp) & 1) ? 64u : 0u;
    const unsigned char* w_tile = p.w + static_cast<size_t>(n0) * k_bytes;
    const unsigned char* x_tile = p.x + static_cast<size_t>(m0) * seg_bytes;
    // A token row's k runs contiguously through the hq_l heads that one source rank returned, then jumps to the
    // next rank's buffer (mode 1); in mode 0 it is contiguous throughout.
    const int seg_tiles = max(static_cast<int>(seg_bytes / kRowBytes), 1);
    const size_t seg_jump = p.mode == 0 ? 0 : static_cast<size_t>(p.s.T_pad - 1) * seg_bytes;
    // The workgroups of a launch move through k in step, and rows lie a power of two apart: left alone, every compute
    // unit of the chip asks for the same few memory channels at the same time (measured: the address path stalled by the
    // cache twice as often, twice the bytes fetched into the L2s).  So the walk over k starts at a different place on
    // every XCD (workgroup i runs on XCD i % 8; the workgroups of one XCD stay together, they share operand panels
    // through its L2) and wraps around; a sum over k does not care where it starts.
    const int rot0 = ragged ? 0 : static_cast<int>((static_cast<int64_t>(blockIdx.x % 8) * k_steps) / 8);
    const unsigned char* const w_start = w_tile + static_cast<size_t>(kt0) * kRowBytes;
    const unsigned char* const x_start = x_tile + static_cast<size_t>(kt0) * kRowBytes + static_cast<size_t>(kt0 / seg_tiles) * seg_jump;
    const int left_start = seg_tiles - kt0 % seg_tiles;
    const int kt_first = kt0 + rot0;
    int ld_kt = 0, ld_left = seg_tiles - kt_first % seg_tiles;   // loads issued so far, and how many stages remain in the segment of the next one
    int wrap_left = k_steps - rot0;                              // stages until the walk is back at the start of its range
    w_tile += static_cast<size_t>(kt_first) * kRowBytes;
    x_tile += static_cast<size_t>(kt_first) * kRowBytes + static_cast<size_t>(kt_first / seg_tiles) * seg_jump;
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
    auto load_one = [&](int j, bool tail) {          // first the token rows, then the weight rows
        unsigned char* dst = lds + (ld_kt % kStages) * kStage + (kLoadRows * wave_s) * kRowBytes;   // (= ld_dst)
        const uint32_t fix = tail ? tail_fix[j % 2] : 0u;
        if (j < kLoadsPerOperand) dma_1k(x_tile, x_off[j] - fix, dst + kOperandBytes + j * 1024);
        else dma_1k(w_tile, w_off[j - kLoadsPerOperand] - fix, dst + (j - kLoadsPerOperand) * 1024);
    };
    auto advance_x = [&]() {              // behind the last token-row load of a stage
        x_tile += kRowBytes;
        if (--ld_left == 0) {             // (a real branch, rarely taken: as selects this is a dozen scalar instructions)
            asm volatile("; next source buffer");
            ld_left = seg_tiles;
            x_tile += seg_jump;
        }
    };
    // LDS address of this wavefront's rows in the stage buffer that the next loads fill
    uint32_t ld_dst = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds + (kLoadRows * wave_s) * kRowBytes));
    uint32_t ld_dst_step = kStage;        // to the other buffer and back
    auto advance_w = [&]() {              // behind the last load of a stage
        ++ld_kt;
        w_tile += kRowBytes;
        if (--wrap_left == 0) {           // (rarely taken, a real branch)
            asm volatile("; back to the start of the k range");
            w_tile = w_start;
            x_tile = x_start;
            ld_left = left_start;
        }
        ld_dst += ld_dst_step;
        ld_dst_step = 0u - ld_dst_step;
    };
    // The same load in two statements, for the loop of the 16-clock MFMAs, where the single wavefront of a SIMD keeps the
    // matrix pipe fed only if no more than one other instruction sits between two MFMAs: the LDS destination into M0
    // (one scalar addition; the MFMA behind it is the wait state the load needs), then, one MFMA later, the load.
    // Nothing else in this kernel writes M0 between the two (the compiler has no use of its own for it here).
    auto set_m0 = [&]<int j>() {
        constexpr int imm = j < kLoadsPerOperand ? kOperandBytes + j * 1024 : (j - kLoadsPerOperand) * 1024;
        const uint32_t dst = ld_dst;
        asm volatile("s_add_u32 m0, %0, %1" :: "s"(dst), "n"(imm) : "scc");
    };
    auto issue_load = [&]<int j>(bool tail) {
        constexpr bool is_x = j < kLoadsPerOperand;
        constexpr int jj = is_x ? j : j - kLoadsPerOperand;
        const uint32_t off = (is_x ? x_off[jj] : w_off[jj]) - (tail ? tail_fix[j % 2] : 0u);
        const unsigned char* base = scalar_ptr(is_x ? x_tile : w_tile);
        asm volatile("global_load_lds_dwordx4 %0, %1" :: "v"(off), "s"(base) : "memory");
    };

    // ---- operand reads: tiles of 16 rows; this wavefront's weight rows and token rows in a stage buffer
    const int a_base = (wn * kWaveRows) * kRowBytes;
    const int b_base = kOperandBytes + (wm * kWaveRows) * kRowBytes;

    // accumulators: 8 x 8 tiles of 16 x 16 per wavefront, 256 registers
    constexpr int kAT = 8;
    f32x4 acc[kAT][kAT];
#pragma unroll
    for (int nt = 0; nt < kAT; ++nt)
#pragma unroll
        for (int mt = 0; mt < kAT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[nt][mt][r] = 0.f;

    // the first two stages are requested (the last one of a short k with its half-row fix), stage 0 has landed everywhere
    auto prologue = [&]() {
        for (int t = 0; t < kStages && t < k_steps; ++t) {
            const bool tail = ragged && t == k_steps - 1;
#pragma unroll
            for (int j = 0; j < kLoadsPerStage; ++j) load_one(j, tail);
            advance_x();
            advance_w();
        }
        if (k_steps >= kStages) __builtin_amdgcn_s_waitcnt(wait_imm(kLoadsPerStage, kNoLgkm));
        else __builtin_amdgcn_s_waitcnt(wait_imm(0, kNoLgkm));
        asm volatile("s_barrier" ::: "memory");
    };
    // The stage loop.  kLoadMode 0: no loads (the last two stages), 1: the loads of the stage after next follow the
    // meeting, 2: the same with the half-row fix (that stage is a half-filled last one).
    auto run_stages = [&](auto&& stage) {
        int st = 0;
        const int n_plain = k_steps - kStages - (ragged ? 1 : 0);
        for (; st < n_plain; ++st) stage.template operator()<1>(st);
        if constexpr (kFp8) {
            if (ragged && st + kStages < k_steps) {
                stage.template operator()<2>(st);
                ++st;
            }
        }
        for (; st < k_steps; ++st) stage.template operator()<0>(st);
    };

    // Operands are read from LDS one MFMA k step (a "slice": 32 bytes of every row for bf16, 64 for FP8) ahead of the
    // MFMAs that use them, into the other of two register sets, one read behind an MFMA, in the order in which the
    // MFMAs of the coming slice need them: the matrix pipe never waits behind a burst of reads (with one wavefront per
    // SIMD nothing else would feed it meanwhile).  The workgroup meets once per stage, in front of the stage's last
    // slice: by then a wavefront holds that slice in registers (it is done with the stage's buffer) and its loads of
    // the next stage have landed.  Behind the meeting the first slice of the next stage is read and the stage after
    // next is requested into the buffer just left, one load behind every MFMA.
    if constexpr (!kFp8) {
        // v_mfma_f32_16x16x32_bf16 (at the chip's power limit it sustains about 15 % more than the 32x32x16 form: it
        // reads and writes a quarter of the accumulator registers per MFMA for half the work).  A slice is 32 k, half
        // a stage: lane -> row lane % 16 of a 16-row tile, piece 4 slice + lane / 16 of its 128-byte row; eight tiles
        // of either operand per wavefront, 64 MFMAs per slice.
        const int r16 = lane & 15, kg = lane >> 4;
        int rd[2];
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) rd[sl] = r16 * kRowBytes + (((4 * sl + kg) ^ ((r16 >> 1) & 7)) << 4);
        u32x4 a[2][kAT], b[2][kAT];   // [set]
        // read r of a slice into set S, in the order of first use by MFMA (i, j) = (I / 8, I % 8): a[0], b[0..7], a[1..7]
        auto read_one = [&]<int r, int S>(const unsigned char* base, int sl) {
            if constexpr (r == 0) a[S][0] = *reinterpret_cast<const u32x4*>(base + a_base + rd[sl]);
            else if constexpr (r <= kAT) b[S][r - 1] = *reinterpret_cast<const u32x4*>(base + b_base + (r - 1) * 16 * kRowBytes + rd[sl]);
            else a[S][r - kAT] = *reinterpret_cast<const u32x4*>(base + a_base + (r - kAT) * 16 * kRowBytes + rd[sl]);
        };
        // the 64 MFMAs of one slice on set S; the 16 reads of (rd_base, rd_sl) into the other set behind MFMAs 0, 4, 8,
        // ... (kDense: 0, 3, ..., 45, so that they are back before the slice ends); kLoadMode > 0: the 16 loads of the
        // stage after next, each in two slots
        auto slice = [&]<int S, bool kDense, int kLoadMode>(const unsigned char* rd_base, int rd_sl) {
            [&]<int... I>(std::integer_sequence<int, I...>) {
                (([&]() {
                     constexpr int i = I / kAT, j = I % kAT;
                     mfma_16x16x32(acc[i][j], a[S][i], b[S][j]);
                     if constexpr (kDense) {
                         if constexpr (I % 3 == 0 && I / 3 < 2 * kAT) read_one.template operator()<I / 3, 1 - S>(rd_base, rd_sl);
                     } else {
                         if constexpr (I % 4 == 0) read_one.template operator()<I / 4, 1 - S>(rd_base, rd_sl);
                     }
                     if constexpr (kLoadMode > 0) {   // load j: M0 behind MFMA 4 j + 1, the load behind MFMA 4 j + 2
                         if constexpr (I % 4 == 1) set_m0.template operator()<I / 4>();
                         if constexpr (I % 4 == 2) issue_load.template operator()<I / 4>(kLoadMode == 2);
                         if constexpr (I == 4 * kLoadsPerOperand - 1) advance_x();   // (scalar work, in slots of its own)
                         if constexpr (I == kAT * kAT - 1) advance_w();
                     }
                     __builtin_amdgcn_sched_barrier(0);
                 }()),
                 ...);
            }(std::make_integer_sequence<int, kAT * kAT>{});
        };
        prologue();
        [&]<int... R>(std::integer_sequence<int, R...>) {
            (read_one.template operator()<R, 0>(lds, 0), ...);
        }(std::make_integer_sequence<int, 2 * kAT>{});
        auto stage = [&]<int kLoadMode>(int st) {
            // (where two copies of this body meet, the compiler moves accumulators between registers; the wait states
            // an MFMA needs behind such a move are put here, since it cannot know that one follows)
            asm volatile("s_nop 4" ::: "memory");
            slice.template operator()<0, true, 0>(lds + (st % kStages) * kStage, 1);
            // this wavefront is done with the buffer, and its loads of the next stage have landed
            __builtin_amdgcn_s_waitcnt(wait_imm(0, 0));
            asm volatile("s_barrier" ::: "memory");
            // (behind the last stage: stale data, not used)
            slice.template operator()<1, false, kLoadMode>(lds + ((st + 1) % kStages) * kStage, 0);
        };
        run_stages(stage);
        mfma_settle();
    } else {
        // v_mfma_scale_f32_16x16x128_f8f6f4 with unit block scales: a stage (128 bytes of a row) is one MFMA k step,
        // 64 MFMAs of 32 clocks; lane -> row lane % 16 of a 16-row tile, pieces 2 (lane / 16) and 2 (lane / 16) + 1 of
        // its row (which k a lane holds does not matter as long as both operands agree).  Registers hold the eight token
        // tiles of the stage (b, 64 registers) and eight weight tiles (a, 64): rows i = 0..3 of the MFMA grid fetch
        // weight tiles 4..7 of the stage, the workgroup meets in front of row 4 (all of the stage's operands are in
        // registers or on their way, the next stage has landed), rows 4..7 fetch weight tiles 0..3 of the next stage and
        // request the stage after next, and token tile j of the next stage is fetched right behind MFMA (7, j), the
        // last one that uses its registers, eight MFMAs ahead of the first one that needs it.
        const int r16 = lane & 15, kg = lane >> 4;
        int rd[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) rd[h] = r16 * kRowBytes + (((2 * kg + h) ^ ((r16 >> 1) & 7)) << 4);
        i32x8 a[kAT], b[kAT];
        int unit_scale;   // E8M0 code of 1.0, in a vector register as the instruction wants it
        asm volatile("v_mov_b32 %0, 127" : "=v"(unit_scale));
        auto join = [](u32x4 lo, u32x4 hi) -> i32x8 {
            return i32x8{static_cast<int>(lo[0]), static_cast<int>(lo[1]), static_cast<int>(lo[2]), static_cast<int>(lo[3]),
                         static_cast<int>(hi[0]), static_cast<int>(hi[1]), static_cast<int>(hi[2]), static_cast<int>(hi[3])};
        };
        auto read_a = [&]<int i>(const unsigned char* base) {
            const unsigned char* row = base + a_base + i * 16 * kRowBytes;
            a[i] = join(*reinterpret_cast<const u32x4*>(row + rd[0]), *reinterpret_cast<const u32x4*>(row + rd[1]));
        };
        auto read_b = [&]<int j>(const unsigned char* base) {
            const unsigned char* row = base + b_base + j * 16 * kRowBytes;
            b[j] = join(*reinterpret_cast<const u32x4*>(row + rd[0]), *reinterpret_cast<const u32x4*>(row + rd[1]));
        };
        // (assembly with the accumulator tied in place, as for bf16 above)
        auto mfma = [&](f32x4& d, const i32x8& av, const i32x8& bv) {
            asm volatile("v_mfma_scale_f32_16x16x128_f8f6f4 %0, %1, %2, %0, %3, %3 op_sel_hi:[0,0,0]"
                         : "+a"(d) : "v"(av), "v"(bv), "v"(unit_scale));
        };
        prologue();
        [&]<int... R>(std::integer_sequence<int, R...>) {
            (read_b.template operator()<R>(lds), ...);
        }(std::make_integer_sequence<int, kAT>{});
        [&]<int... R>(std::integer_sequence<int, R...>) {
            (read_a.template operator()<R>(lds), ...);
        }(std::make_integer_sequence<int, kAT / 2>{});
        auto stage = [&]<int kLoadMode>(int st) {
            const unsigned char* cur = lds + (st % kStages) * kStage;
            const unsigned char* nxt = lds + ((st + 1) % kStages) * kStage;
            asm volatile("s_nop 4" ::: "memory");   // (accumulator moves between two copies of this body, see above)
            if (kLoadMode == 0 && ragged && st == k_steps - 1) {
                // a half-filled last stage: the upper 64 bytes of its rows repeat the lower ones (see the loads); the
                // lanes that hold them multiply by zero
#pragma unroll
                for (int j = 0; j < kAT; ++j)
#pragma unroll
                    for (int e = 0; e < 8; ++e) b[j][e] = kg >= 2 ? 0 : b[j][e];
                asm volatile("s_nop 4" ::: "memory");
            }
            [&]<int... I>(std::integer_sequence<int, I...>) {
                (([&]() {
                     constexpr int i = I / kAT, j = I % kAT;
                     if constexpr (I == kAT * kAT / 2) {
                         // this wavefront is done with the buffer, and its loads of the next stage have landed
                         __builtin_amdgcn_s_waitcnt(wait_imm(0, 0));
                         asm volatile("s_barrier" ::: "memory");
                     }
                     mfma(acc[i][j], a[i], b[j]);
                     if constexpr (i < kAT / 2 && j == 0) read_a.template operator()<i + kAT / 2>(cur);
                     if constexpr (i >= kAT / 2 && j == 1) read_a.template operator()<i - kAT / 2>(nxt);   // (behind the last stage: stale, unused)
                     if constexpr (i == kAT - 1) read_b.template operator()<j>(nxt);
                     if constexpr (kLoadMode > 0 && i >= kAT / 2) {   // 16 loads in the 32 slots behind the meeting: M0, then the load
                         constexpr int slot = I - kAT * kAT / 2;
                         if constexpr (slot % 2 == 0) set_m0.template operator()<slot / 2>();
                         else issue_load.template operator()<slot / 2>(kLoadMode == 2);
                         if constexpr (slot == 2 * kLoadsPerOperand - 1) advance_x();
                         if constexpr (slot == 2 * kLoadsPerStage - 1) advance_w();
                     }
                     __builtin_amdgcn_sched_barrier(0);
                 }()),
                 ...);
            }(std::make_integer_sequence<int, kAT * kAT>{});
        };
        run_stages(stage);
        mfma_settle();
    }

    // ---- result.  A lane holds runs of four consecutive features of one token: acc[i][j] is features
    // 16 i + 4 (lane / 16) .. + 3 of token 16 j + lane % 16.
    int tid_e = threadIdx.x;
    asm volatile("" : "+v"(tid_e));
    const int lane_e = tid_e & 63;
    constexpr int kTokStep = 16;
    constexpr int kQuads = kAT;
    const int tok_lane = lane_e & 15;
    auto quad_feature = [&](int q) { return 16 * q + 4 * (lane_e >> 4); };
    auto quad_value = [&](int q, int t, int e) -> float { return acc[q][t][e]; };
    const int f_wave = n0 + wn * (kTile / kWavesN);     // first feature of this wavefront; its features lie in one head
    // The bf16 result goes through LDS (the stage buffers are free by now): a wavefront lays its 128 tokens x 128
    // features down as rows of 256 bytes (pitch 272: the 8-byte writes of 16 token rows then spread over all banks),
    // reads them back 16 bytes per lane and stores whole rows - 256 contiguous bytes per token instead of the 8-byte
    // pieces the accumulator layout would give (those cost 4 % of the kernel).  A wavefront reads only what it wrote
    // itself, so the workgroup does not meet; what other wavefronts may still be reading there is discarded anyway
    // (the last stage's look-ahead reads).
    unsigned char* stg = lds + wave * kStagingWave;
    auto stage_result = [&]() {
#pragma unroll
        for (int t = 0; t < kAT; ++t) {
            const int tok = t * kTokStep + tok_lane;
            const int m = m0 + wm * kWaveRows + tok;
            float row_scale = 1.f;
            if constexpr (kFp8) row_scale = m < p.M ? p.xs[m] : 0.f;
#pragma unroll
            for (int q = 0; q < kQuads; ++q) {
                const int f = quad_feature(q);
                f32x4 col_scale = {1.f, 1.f, 1.f, 1.f};
                if constexpr (kFp8) col_scale = *reinterpret_cast<const f32x4*>(p.ws + f_wave + f);
                bf16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float y = m < p.M ? quad_value(q, t, e) : 0.f;   // rows M .. M_out - 1 of the result are zeros
                    if constexpr (kFp8) y = y * row_scale * col_scale[e];
                    v[e] = static_cast<__bf16>(y);
                }
                *reinterpret_cast<u32x2*>(stg + tok * kStagingPitch + f * 2) = __builtin_bit_cast(u32x2, v);
            }
        }
    };
    auto store_rows = [&](uint16_t* dst_row0, size_t row_stride) {   // dst_row0: feature f_wave of token row 0
#pragma unroll 8
        for (int r = 0; r < kWaveRows / 4; ++r) {
            const int tok = 4 * r + (lane_e >> 4);
            const int m = m0 + wm * kWaveRows + tok;
            if (m >= p.M_out) continue;
            const u32x4 v = *reinterpret_cast<const u32x4*>(stg + tok * kStagingPitch + (lane_e & 15) * 16);
            *reinterpret_cast<u32x4*>(dst_row0 + static_cast<size_t>(m) * row_stride + (lane_e & 15) * 8) = v;
        }
    };
    if constexpr (kSplit) {   // this k range's fp32 sums, [split][token][feature]; proj_finish adds the ranges and does the layout
        float* base = p.partial + static_cast<size_t>(split) * (p.M_out - p.m_base) * p.N + f_wave;   // [split][row - m_base][feature]
#pragma unroll
        for (int t = 0; t < kAT; ++t) {
            const int m = m0 + wm * (kTile / kWavesM) + t * kTokStep + tok_lane;
            if (m >= p.M) continue;   // rows past the last token are zeros in the result and are not read
            float* row = base + static_cast<size_t>(m - p.m_base) * p.N;
#pragma unroll
            for (int q = 0; q < kQuads; ++q)
                *reinterpret_cast<f32x4*>(row + quad_feature(q)) =
                    f32x4{quad_value(q, t, 0), quad_value(q, t, 1), quad_value(q, t, 2), quad_value(q, t, 3)};
        }
        return;
    }
    stage_result();
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

// The grid is persistent: one workgroup per compute unit walks the launch's work items (output tile, k range) with
// stride gridDim.x, so a compute unit goes from one tile to the next without waiting for a workgroup to be scheduled
// (ten rounds of tiles at the 70B shape).  Item i runs on the XCD workgroup i % gridDim.x was placed on; with a grid
// that is a multiple of 8 an XCD keeps seeing neighbouring tiles, which share operand panels through its L2.
template <bool kFp8, bool kSplit>
__global__ __launch_bounds__(kGemmThreads) void proj_gemm_kernel(GemmParams p) {
    for (int item = blockIdx.x; item < p.items; item += gridDim.x) {
        proj_gemm_tile<kFp8, kSplit>(p, item);
        // the next item's loads go where other wavefronts may still be reading their staged result rows
        __builtin_amdgcn_s_waitcnt(wait_imm(kNoVm, 0));
        asm volatile("s_barrier" ::: "memory");
    }
}

template <bool kFp8>
hipError_t launch(const GemmParams& p, hipStream_t st) {
    const int64_t items = static_cast<int64_t>(p.N / kTile) * p.m_tiles * p.k_splits;
    if (items == 0) return hipSuccess;
    if (items > 0x7FFFFFFF) return hipErrorInvalidValue;
    GemmParams q = p;
    q.items = static_cast<int>(items);
    int cus = 0, device = 0;   // one workgroup fits a compute unit (registers, LDS)
    hipError_t e = hipGetDevice(&device);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
    if (e != hipSuccess) return e;
    const unsigned grid = static_cast<unsigned>(items < cus ? items : cus);
    if (p.k_splits > 1) {
        proj_gemm_kernel<kFp8, true><<<grid, kGemmThreads, kGemmLds, st>>>(q);
        return hipGetLastError();
    }
    proj_gemm_kernel<kFp8, false><<<grid, kGemmThreads, kGemmLds, st>>>(q);
    return hipGetLastError();
}

// How a product is laid over the 256 compute units.  The grid walks whole output tiles; when their number is no
// multiple of 256 (or below it) the last round would leave most of the chip idle, so the trailing token tiles can
// instead be split over k: `unsplit_tiles` leading token tiles (256 rows each) are done whole, the rest in `splits`
// ranges of k whose fp32 sums go to the caller's workspace and are added by the finishing kernel.  Chosen by a rough
// model of the launches - a workgroup walks all of k of a tile at about 6.5 TFLOP/s (12.5 over FP8 operands),
// work items beyond one per compute unit queue up in rounds, every range adds fp32 partial results that are written and
// read back.  Ranges are at least 8 k stages long.  splits == 1: everything whole.
struct GemmPlan {
    int unsplit_tiles, splits;
};
GemmPlan plan_gemm(int M_out, int N, int K, bool fp8) {
    const int n_tiles = N / kTile, m_tiles = (M_out + kTile - 1) / kTile;
    GemmPlan best = {m_tiles, 1};
    if (n_tiles == 0 || m_tiles == 0) return best;
    const double walk = 2.0 * kTile * kTile * static_cast<double>(K) / (fp8 ? 12.5e12 : 6.5e12);   // one workgroup over all of k
    auto rounds = [](int64_t items) { return static_cast<double>((items + 255) / 256); };
    const int by_length = K / (fp8 ? 64 : 32) / 16;
    double t_best = rounds(static_cast<int64_t>(n_tiles) * m_tiles) * walk;
    const double t_whole = t_best;
    for (int ma = 0; ma < m_tiles; ++ma) {
        const int64_t tiles_b = static_cast<int64_t>(n_tiles) * (m_tiles - ma);
        const double rows_b = static_cast<double>(M_out - ma * kTile);
        const double partial = 2.0 * rows_b * N * sizeof(float) / 3.2e12;   // written once, read once
        const double t_a = ma > 0 ? rounds(static_cast<int64_t>(n_tiles) * ma) * walk + 3.0e-6 : 0.0;
        for (int sp = 2; sp <= 16 && sp <= by_length; ++sp) {
            const double t = t_a + rounds(tiles_b * sp) / sp * walk + sp * partial + 5.0e-6;
            if (t < t_best && t < 0.97 * t_whole) {
                t_best = t;
                best = {ma, sp};
            }
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
    const GemmPlan pl = plan_gemm(M_out, N, K, fp8);
    return pl.splits == 1 ? 0 : static_cast<size_t>(pl.splits) * (M_out - pl.unsplit_tiles * kTile) * N * sizeof(float);
}

// runs the product as planned when the workspace holds the partial results, else in whole tiles
static hipError_t run_gemm(GemmParams& p, void* workspace, size_t workspace_bytes, hipStream_t st) {
    const bool fp8 = p.xs != nullptr;
    const int m_tiles = (p.M_out + kTile - 1) / kTile;
    p.k_splits = 1;
    p.partial = nullptr;
    p.m_base = 0;
    p.m_tiles = m_tiles;
    const GemmPlan pl = plan_gemm(p.M_out, p.N, p.K, fp8);
    const size_t need = proj_gemm_workspace(p.M_out, p.N, p.K, fp8);
    if (need == 0 || need > workspace_bytes || !workspace) return fp8 ? launch<true>(p, st) : launch<false>(p, st);
    if (pl.unsplit_tiles > 0) {
        p.m_tiles = pl.unsplit_tiles;
        const hipError_t e = fp8 ? launch<true>(p, st) : launch<false>(p, st);
        if (e != hipSuccess) return e;
    }
    p.m_base = pl.unsplit_tiles * kTile;
    p.m_tiles = m_tiles - pl.unsplit_tiles;
    p.k_splits = pl.splits;
    p.partial = static_cast<float*>(workspace);
    const hipError_t e = fp8 ? launch<true>(p, st) : launch<false>(p, st);
    if (e != hipSuccess) return e;
    return launch_proj_finish(p.partial, p.k_splits, p.M_out - p.m_base, p.c, p.M, p.M_out, p.N, p.mode, p.s, p.xs, p.ws, st,
                              p.m_base);
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
