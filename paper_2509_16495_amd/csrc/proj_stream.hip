// The two projections next to the exchange (Algorithm 1: qkv = embed * W_qkv, embed = attn_o * W_o) for the few
// tokens of a decode step (Algorithm 2, the small-batch side of the threshold).  With up to 64 token rows the product
// is bound by reading the weight matrix once from HBM, not by the matrix cores, so the kernel is organised around
// that stream:
//
//   * 256 workgroups of eight wavefronts, one per compute unit, each owning a contiguous block of output features
//     (N / 256 rows, so every compute unit reads the same number of weight bytes) and walking it in tiles of 16;
//   * the eight wavefronts of a workgroup split k: wavefront w multiplies k slice w of every tile.  Its slice of the
//     token rows (16 TB tokens x KWB steps of 128 bytes of k: 64 bf16 or 128 FP8 elements; TB KWB <= 16) stays in
//     128 registers for the whole kernel in MFMA operand layout, so the only traffic of the main loop is the weights;
//   * weights arrive by direct-to-LDS loads (1 KiB per instruction: eight rows x 128 bytes, whole cache lines, marked
//     non-temporal: they are used once) into a ring private to the wavefront - no workgroup barrier in the stream, a
//     wavefront waits for its own loads by count, seven or eight steps of 2 KiB in flight - and are read back as
//     MFMA A operands (two v_mfma_f32_16x16x32_bf16 per step and token block, or one
//     v_mfma_scale_f32_16x16x128_f8f6f4 over FP8 codes); the 128 bytes of a row keep their eight 16-byte pieces at
//     positions piece ^ (row / 2) % 8, which makes those reads conflict-free;
//   * the token rows are requested behind the first steps of weights and waited for piecewise inside the first tile,
//     so the stream is already running while they arrive (every workgroup reads all of them: 64 MB through the L2s at
//     16 tokens and k = 8192, which is what a 16-token call costs over a 1-token call);
//   * per tile the eight partial 16 x 16 TB results meet in LDS and are summed in wavefront order (bitwise
//     reproducible), multiplied by the token's and the feature's scale when the operands are FP8 codes, rounded once
//     to bf16 and stored where the pack / unpack would have put them.
//
// When the token rows do not fit the registers of eight wavefronts (more than 16 bf16 or 32 FP8 tokens at k = 8192), k is split
// over `kg` workgroups as well; those write fp32 partial results to a caller-provided workspace and a small second
// kernel sums them in group order and does the rounding and the layout.
#include "internal.h"

#include <utility>

namespace shiftattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int kSWaves = 8, kSThreads = 64 * kSWaves;
constexpr int kSGrid = 256;                        // workgroups: one per compute unit
constexpr int kStepRowBytes = 128;                 // bytes of a weight row per step of a wavefront: 64 bf16 or 128 FP8 k
constexpr int kStepBytes = 16 * kStepRowBytes;     // 16 weight rows
constexpr int kHeadDim = 128;
#define SHIFTATTN_STREAM_HINT " nt"   // weights are read once: non-temporal

struct StreamParams {
    const unsigned char* __restrict__ w;   // [N][K] bf16 or FP8 E4M3 codes
    const unsigned char* __restrict__ x;   // token rows, see mode
    uint16_t* __restrict__ c;              // bf16 result (kg == 1)
    float* __restrict__ partial;           // [kg][16 TB][N] fp32 (kg > 1)
    const float* __restrict__ xs;          // FP8 products: one scale per token row ...
    const float* __restrict__ ws;          // ... and one per output feature (nullptr: none)
    int M, M_out, N, K;                    // M token rows exist, rows M .. M_out - 1 of the result are zeros
    int mode;                              // 0: x dense [M][K], result into the send buffers; 1: x gathered from the
                                           // receive buffers (k = (p hq_l + j) 128 + e), result dense [M][N]
    int kg;                                // workgroups that share a block of features (k groups)
    int rows_per_block;                    // features per block, a multiple of 4
    XchgShape s;
};

__device__ inline bf16x8 frag(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Four bf16 results of token t, features f .. f + 3 (one head, col = f % 128), to their place(s):
// mode 1: out[t][f]; mode 0: the send buffer(s) of the rank(s) owning the head (Sec. 3.2.1: fused q|k|v exchange,
// KV replication when there are fewer KV heads than ranks).
__device__ inline void store4(const StreamParams& p, int t, int f, u32x2 v) {
    if (p.mode == 1) {
        *reinterpret_cast<u32x2*>(p.c + static_cast<size_t>(t) * p.N + f) = v;
        return;
    }
    const XchgShape& s = p.s;
    const int head = f / kHeadDim, col = f % kHeadDim;
    const size_t row_stride = static_cast<size_t>(s.hq_l + 2 * s.hkv_l) * kHeadDim;
    const size_t buf_stride = static_cast<size_t>(s.T_pad) * row_stride;
    uint16_t* row = p.c + static_cast<size_t>(t) * row_stride + col;
    if (head < s.h) {
        const int dest = head / s.hq_l, local = head - dest * s.hq_l;
        *reinterpret_cast<u32x2*>(row + dest * buf_stride + local * kHeadDim) = v;
        return;
    }
    const bool is_v = head >= s.h + s.h_kv;
    const int g = head - s.h - (is_v ? s.h_kv : 0);
    const int slot0 = s.hq_l + (is_v ? s.hkv_l : 0);
    if (s.h_kv >= s.P) {
        const int dest = g / s.hkv_l, local = slot0 + (g - dest * s.hkv_l);
        *reinterpret_cast<u32x2*>(row + dest * buf_stride + local * kHeadDim) = v;
    } else {
        for (int dest = 0; dest < s.P; ++dest)
            if (static_cast<int>((static_cast<int64_t>(dest) * s.h_kv) / s.P) == g)
                *reinterpret_cast<u32x2*>(row + dest * buf_stride + slot0 * kHeadDim) = v;
    }
}

__device__ inline u32x2 round4(f32x4 v) {
    bf16x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = static_cast<__bf16>(v[e]);
    return __builtin_bit_cast(u32x2, r);
}

// TB: token blocks of 16; KWB: steps (128 bytes of a weight row: 64 bf16 or 128 FP8 k) in a wavefront's k slice;
// kStages: steps in a wavefront's ring; kFp8: both operands are FP8 E4M3 codes (one v_mfma_scale_f32_16x16x128_f8f6f4
// with unit block scales per step and token block instead of two bf16 MFMAs; the token's and the feature's scale
// multiply the sum before it is rounded - or in the finishing kernel when k is split over workgroups)
template <int TB, int KWB, int kStages, bool kFp8>
__global__ __launch_bounds__(kSThreads) void proj_stream_kernel(StreamParams p) {
    constexpr int kElem = kFp8 ? 1 : 2;
    constexpr int kStepK = kStepRowBytes / kElem;
    static_assert(TB * KWB <= 16, "the token slice of a wavefront fits 128 registers");
    constexpr int kXLoads = TB * KWB * 2;          // 16-byte loads of token data per lane
    static_assert(2 * (kStages - 1) + kXLoads + 2 <= 62, "outstanding loads fit the counter");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, grp = lane >> 4;
    const int cgrp = blockIdx.x % p.kg, rb = blockIdx.x / p.kg;
    const int row_begin = rb * p.rows_per_block;
    const int row_end = min(p.N, row_begin + p.rows_per_block);
    if (row_begin >= row_end) return;   // the whole workgroup
    const int n_tiles = (row_end - row_begin + 15) >> 4;
    const int total = n_tiles * KWB;    // steps of this wavefront
    const int k0 = (cgrp * kSWaves + wave) * (KWB * kStepK);
    const size_t k_bytes = static_cast<size_t>(p.K) * kElem;
    const uint32_t ring = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds)) + wave * (kStages * kStepBytes);
    unsigned char* ring_ptr = lds + wave * (kStages * kStepBytes);
    f32x4* red = reinterpret_cast<f32x4*>(lds + kSWaves * kStages * kStepBytes);   // [wavefront][TB][lane]

    // ---- the weight stream: step (tile, st) is rows 16 tile .. + 15 of the block, k0 + 64 st .. + 63
    auto scalar_ptr = [](const unsigned char* ptr) -> const unsigned char* {
        const uint64_t a = reinterpret_cast<uint64_t>(ptr);
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
        return reinterpret_cast<const unsigned char*>((static_cast<uint64_t>(hi) << 32) | lo);
    };
    // 1 KiB from a wavefront-uniform base + a 32-bit byte offset per lane into LDS at dst (uniform); waited for by count
    auto dma_1k = [&](const unsigned char* base, uint32_t lane_off, uint32_t dst) {
        // (M0 is reserved by the compiler - it sets it right before each use of its own and keeps no value in it, and
        // rejects it on a clobber list - so writing it here needs no clobber.)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" SHIFTATTN_STREAM_HINT
                     :: "s"(dst), "v"(lane_off), "s"(scalar_ptr(base)) : "memory");
    };
    // Every vector memory load of this wavefront is issued by the code below, in a known order (kStages - 1 steps of
    // weights, the token rows, then a step of weights per step computed), and loads return in order.
    uint32_t off[2];   // this lane's piece of instruction i: row 8 i + lane / 8, position lane % 8 holds piece position ^ key(row)
    auto tile_offsets = [&](int tile) {   // rows past the end of the block re-read its last row; they are not stored
        const int row0 = row_begin + 16 * tile;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = 8 * i + (lane >> 3);
            const int row = min(row0 + r, row_end - 1) - row0;
            off[i] = static_cast<uint32_t>(static_cast<size_t>(row) * k_bytes + (((lane & 7) ^ ((r >> 1) & 7)) << 4));
        }
    };
    int rq_g = 0, rq_st = 0, rq_tile = 0, rq_slot = 0;   // the next step to request
    const unsigned char* rq_base = p.w + static_cast<size_t>(row_begin) * k_bytes + static_cast<size_t>(k0) * kElem;
    auto request = [&]() {
        const uint32_t dst = ring + rq_slot * kStepBytes;
#pragma unroll
        for (int i = 0; i < 2; ++i) dma_1k(rq_base, off[i], dst + 1024 * i);
        ++rq_g;
        rq_slot = rq_slot + 1 == kStages ? 0 : rq_slot + 1;
        if (++rq_st == KWB) {
            rq_st = 0;
            ++rq_tile;
            rq_base += 16 * k_bytes - (KWB - 1) * kStepRowBytes;
            if (rq_tile < n_tiles) tile_offsets(rq_tile);
        } else {
            rq_base += kStepRowBytes;
        }
    };
    tile_offsets(0);
    for (int g = 0; g < kStages - 1 && g < total; ++g) request();

    // ---- this wavefront's slice of the token rows, as B operands: lane (token l16, k group grp), requested in the
    // order the first tile uses them, so that the first tile starts while most of them are still on their way.  Rows
    // past the last token re-read the last one: a token is a column of the product, and those columns are not stored.
    u32x4 xr[TB][KWB * 2];
#pragma unroll
    for (int b = 0; b < KWB * 2; ++b) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            const int t_src = min(16 * tb + l16, p.M - 1);
            // the 16 bytes of token t_src this lane multiplies with weight piece (b % 2 ? second : first) of step b / 2:
            // bf16: k block b (32 k), its k group grp; FP8: step b / 2, the lane's 32 k in two halves
            const int k = kFp8 ? k0 + 128 * (b >> 1) + 32 * grp + 16 * (b & 1) : k0 + 32 * b + 8 * grp;
            const unsigned char* src;
            if (p.mode == 0) {
                src = p.x + (static_cast<size_t>(t_src) * p.K + k) * kElem;
            } else {
                const int seg = p.s.hq_l * kHeadDim;   // contiguous k of a token row in one receive buffer
                const int ps = k / seg, rem = k - ps * seg;
                src = p.x + ((static_cast<size_t>(ps) * p.s.T_pad + t_src) * seg + rem) * kElem;
            }
            asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(xr[tb][b]) : "v"(src) : "memory");
        }
    }

    // ---- operand reads: row l16, piece 4 kb + grp (bf16: k group grp of k block kb) or 2 grp + kb (FP8: the halves of
    // the lane's 32 k) at position piece ^ key(row)
    int rd[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
        rd[kb] = l16 * kStepRowBytes + ((((kFp8 ? 2 * grp + kb : 4 * kb + grp)) ^ ((l16 >> 1) & 7)) << 4);

    int g = 0, slot = 0;
    // One step: the slot read one step ago is free, so the step kStages - 1 ahead is requested into it; then the wait
    // until this step (and, in the first tile, this step's token data) has landed - a wait names how many of the
    // youngest loads may still be outstanding.  kFirst: a step of the first tile; its counts are constants when the
    // wavefront has at least kStages - 1 + KWB steps (`ahead`: every step of the first tile requests one), and a
    // wavefront with fewer steps waits for everything instead.
    const bool ahead = total >= kStages - 1 + KWB;
    f32x4 acc[TB];
    auto step = [&]<bool kFirst, int st>() {
        if constexpr (kFirst) {
            if (ahead || rq_g < total) request();
            if (!ahead) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            constexpr int kIssued = 2 * (kStages - 1) + kXLoads + 2 * (st + 1);
            constexpr int kRing = st < kStages - 1 ? 2 * (st + 1) : kXLoads + 2 * (st + 1);   // this step's last load
            constexpr int kTokens = 2 * (kStages - 1) + 2 * TB * (st + 1);                     // its token data
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kIssued - (kRing > kTokens ? kRing : kTokens)) : "memory");
        } else {
            if (rq_g < total) {
                request();
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * (kStages - 1)) : "memory");
            } else {
                const int younger = total - 1 - g;   // steps requested after this one
#pragma unroll
                for (int y = 0; y < kStages - 1; ++y)
                    if (younger == y) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * y) : "memory");
            }
        }
        if constexpr (kFirst) {
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
                asm volatile("" : "+v"(xr[tb][2 * st]), "+v"(xr[tb][2 * st + 1]));   // used only behind the wait
        }
        const unsigned char* stage = ring_ptr + slot * kStepBytes;
        u32x4 a[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) a[kb] = *reinterpret_cast<const u32x4*>(stage + rd[kb]);
        if constexpr (kFp8) {
            const i32x8 a8 = {static_cast<int>(a[0][0]), static_cast<int>(a[0][1]), static_cast<int>(a[0][2]), static_cast<int>(a[0][3]),
                              static_cast<int>(a[1][0]), static_cast<int>(a[1][1]), static_cast<int>(a[1][2]), static_cast<int>(a[1][3])};
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const u32x4 lo = xr[tb][2 * st], hi = xr[tb][2 * st + 1];
                const i32x8 b8 = {static_cast<int>(lo[0]), static_cast<int>(lo[1]), static_cast<int>(lo[2]), static_cast<int>(lo[3]),
                                  static_cast<int>(hi[0]), static_cast<int>(hi[1]), static_cast<int>(hi[2]), static_cast<int>(hi[3])};
                acc[tb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, acc[tb], 0, 0, 0, 127, 0, 127);
            }
        } else {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int tb = 0; tb < TB; ++tb)
                    acc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag(a[kb]), frag(xr[tb][2 * st + kb]), acc[tb], 0, 0, 0);
        }
        slot = slot + 1 == kStages ? 0 : slot + 1;
        ++g;
    };
    auto do_tile = [&]<bool kFirst>(int tile) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
        [&]<int... st>(std::integer_sequence<int, st...>) {
            (step.template operator()<kFirst, st>(), ...);
        }(std::make_integer_sequence<int, KWB>{});
        // ---- the eight k slices of the tile meet: register r of acc[tb] is feature 4 grp + r of token 16 tb + l16
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();   // the sums of the tile before have been read (bare: no wait for loads in flight)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) red[(wave * TB + tb) * 64 + lane] = acc[tb];
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        if (wave < TB) {
            const int tb = wave;
            f32x4 sum = red[tb * 64 + lane];
#pragma unroll
            for (int w2 = 1; w2 < kSWaves; ++w2) {
                const f32x4 v = red[(w2 * TB + tb) * 64 + lane];
#pragma unroll
                for (int e = 0; e < 4; ++e) sum[e] += v[e];
            }
            const int t = 16 * tb + l16, f = row_begin + 16 * tile + 4 * grp;
            if (f < row_end) {
                if (p.kg > 1) {
                    *reinterpret_cast<f32x4*>(p.partial + (static_cast<size_t>(cgrp) * (16 * TB) + t) * p.N + f) = sum;
                } else if (t < p.M_out) {
                    if constexpr (kFp8) {
                        if (t < p.M) {
                            const float row_scale = p.xs[t];
                            const f32x4 col_scale = *reinterpret_cast<const f32x4*>(p.ws + f);
#pragma unroll
                            for (int e = 0; e < 4; ++e) sum[e] = sum[e] * row_scale * col_scale[e];
                        }
                    }
                    store4(p, t, f, t < p.M ? round4(sum) : u32x2{0u, 0u});
                }
            }
        }
    };
    do_tile.template operator()<true>(0);
    for (int tile = 1; tile < n_tiles; ++tile) do_tile.template operator()<false>(tile);
}

// kg > 1: result[t][f .. f + 3] = sum over the k groups in group order, rounded once
// (row_base: partial row r is row row_base + r of the result)
__global__ __launch_bounds__(256) void proj_stream_finish_kernel(StreamParams p, int t_rows, int row_base) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int quads = p.N / 4;
    if (i >= static_cast<int64_t>(p.M_out - row_base) * quads) return;
    const int r = static_cast<int>(i / quads), f = static_cast<int>(i % quads) * 4;
    const int t = row_base + r;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    if (t < p.M) {
        sum = *reinterpret_cast<const f32x4*>(p.partial + static_cast<size_t>(r) * p.N + f);
        for (int c = 1; c < p.kg; ++c) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(p.partial + (static_cast<size_t>(c) * t_rows + r) * p.N + f);
#pragma unroll
            for (int e = 0; e < 4; ++e) sum[e] += v[e];
        }
        if (p.xs) {   // the scales of FP8 operands, applied as the unsplit kernel applies them
            const float row_scale = p.xs[t];
            const f32x4 col_scale = *reinterpret_cast<const f32x4*>(p.ws + f);
#pragma unroll
            for (int e = 0; e < 4; ++e) sum[e] = sum[e] * row_scale * col_scale[e];
        }
    }
    store4(p, t, f, round4(sum));
}

struct StreamPlan {
    int tb, kwb, kg;   // token blocks of 16, steps per wavefront's k slice, k groups; tb == 0: not served
};

// The largest k slice per wavefront that fits the registers decides how many workgroups must share a block of features.
StreamPlan plan_stream(int M_out, int K, bool fp8) {
    StreamPlan pl = {0, 0, 0};
    const int step_k = kStepRowBytes / (fp8 ? 1 : 2);
    if (M_out < 1 || M_out > 64 || K % (kSWaves * step_k) != 0) return pl;
    const int tb = M_out <= 16 ? 1 : M_out <= 32 ? 2 : 4;
    const int per_wave = K / (kSWaves * step_k);   // steps per wavefront if one workgroup covered all of k
    for (int kwb = 16 / tb; kwb >= 1; kwb /= 2) {
        if (per_wave % kwb != 0) continue;
        const int kg = per_wave / kwb;
        if (kg > 8 || kSGrid % kg != 0) continue;
        pl = {tb, kwb, kg};
        return pl;
    }
    return pl;
}

template <int TB>
constexpr int stream_stages() { return TB == 1 ? 9 : TB == 2 ? 8 : 7; }
template <int TB>
constexpr int stream_lds() { return kSWaves * stream_stages<TB>() * kStepBytes + kSWaves * TB * 64 * 16; }
static_assert(stream_lds<1>() <= 160 * 1024 && stream_lds<2>() <= 160 * 1024 && stream_lds<4>() <= 160 * 1024, "LDS of a compute unit");

template <int TB, int KWB, bool kFp8>
hipError_t launch_stream(const StreamParams& p, hipStream_t st) {
    proj_stream_kernel<TB, KWB, stream_stages<TB>(), kFp8><<<kSGrid, kSThreads, stream_lds<TB>(), st>>>(p);
    return hipGetLastError();
}

template <int TB, int KWB, bool kFp8>
hipError_t init_stream() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&proj_stream_kernel<TB, KWB, stream_stages<TB>(), kFp8>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, stream_lds<TB>());
}

// the instantiated (token blocks, steps per k slice) pairs: X(tb, kwb)
#define SHIFTATTN_STREAM_SHAPES(X) \
    X(1, 16) X(1, 8) X(1, 4) X(1, 2) X(1, 1) X(2, 8) X(2, 4) X(2, 2) X(2, 1) X(4, 4) X(4, 2) X(4, 1)

hipError_t run_stream(StreamParams p, const StreamPlan& pl, void* workspace, hipStream_t st) {
    p.kg = pl.kg;
    p.partial = static_cast<float*>(workspace);
    const int blocks = kSGrid / pl.kg;
    p.rows_per_block = ((p.N + blocks - 1) / blocks + 3) / 4 * 4;
    hipError_t e = hipErrorInvalidValue;
    if (p.xs) {
#define SHIFTATTN_STREAM_LAUNCH(tb_, kwb_) if (pl.tb == tb_ && pl.kwb == kwb_) e = launch_stream<tb_, kwb_, true>(p, st);
        SHIFTATTN_STREAM_SHAPES(SHIFTATTN_STREAM_LAUNCH)
#undef SHIFTATTN_STREAM_LAUNCH
    } else {
#define SHIFTATTN_STREAM_LAUNCH(tb_, kwb_) if (pl.tb == tb_ && pl.kwb == kwb_) e = launch_stream<tb_, kwb_, false>(p, st);
        SHIFTATTN_STREAM_SHAPES(SHIFTATTN_STREAM_LAUNCH)
#undef SHIFTATTN_STREAM_LAUNCH
    }
    return e;
}

}  // namespace

// result = sum over kg partial results [kg][t_rows][N] (fp32) in group order, rounded once, stored with the layout of `mode`
hipError_t launch_proj_finish(const float* partial, int kg, int t_rows, void* c, int M, int M_out, int N, int mode,
                              const XchgShape& s, const float* x_scales, const float* w_scales, hipStream_t st, int row_base) {
    StreamParams p = {};
    p.xs = x_scales;
    p.ws = w_scales;
    p.partial = const_cast<float*>(partial);
    p.c = static_cast<uint16_t*>(c);
    p.M = M;
    p.M_out = M_out;
    p.N = N;
    p.mode = mode;
    p.kg = kg;
    p.s = s;
    const int64_t items = static_cast<int64_t>(M_out - row_base) * (N / 4);
    if (items <= 0) return hipSuccess;
    proj_stream_finish_kernel<<<static_cast<unsigned>((items + 255) / 256), 256, 0, st>>>(p, t_rows, row_base);
    return hipGetLastError();
}

hipError_t proj_stream_init() {
    hipError_t e = hipSuccess;
#define SHIFTATTN_STREAM_INIT(tb_, kwb_)                         \
    if (e == hipSuccess) e = init_stream<tb_, kwb_, false>(); \
    if (e == hipSuccess) e = init_stream<tb_, kwb_, true>();
    SHIFTATTN_STREAM_SHAPES(SHIFTATTN_STREAM_INIT)
#undef SHIFTATTN_STREAM_INIT
    return e;
}

// bytes of workspace the streaming kernel needs for M_out token rows (0: none, or the shape is not served by it)
size_t proj_stream_workspace(int M_out, int N, int K, bool fp8) {
    const StreamPlan pl = plan_stream(M_out, K, fp8);
    return pl.tb == 0 || pl.kg == 1 ? 0 : static_cast<size_t>(pl.kg) * 16 * pl.tb * N * sizeof(float);
}

// served: up to 64 token rows, and either no workspace needed or one of sufficient size given
bool proj_stream_takes(int M_out, int N, int K, bool fp8, size_t workspace_bytes) {
    const StreamPlan pl = plan_stream(M_out, K, fp8);
    return pl.tb != 0 && N % 4 == 0 && proj_stream_workspace(M_out, N, K, fp8) <= workspace_bytes;
}

// x_scales / w_scales: nullptr for bf16 operands, the row scales of FP8 E4M3 codes otherwise
hipError_t launch_qkv_proj_stream(const void* x, const void* w_qkv, void* send, int d_model, const XchgShape& s,
                                  const float* x_scales, const float* w_scales, void* workspace, hipStream_t st) {
    StreamParams p = {};
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
    const StreamPlan pl = plan_stream(p.M_out, p.K, x_scales != nullptr);
    const hipError_t e = run_stream(p, pl, workspace, st);
    if (e != hipSuccess || pl.kg == 1) return e;
    return launch_proj_finish(static_cast<const float*>(workspace), pl.kg, 16 * pl.tb, send, p.M, p.M_out, p.N, 0, s, x_scales, w_scales, st);
}

hipError_t launch_o_proj_stream(const void* recv, const void* w_o, void* out, int d_model, const XchgShape& s,
                                const float* a_scales, const float* w_scales, void* workspace, hipStream_t st) {
    StreamParams p = {};
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
    const StreamPlan pl = plan_stream(p.M_out, p.K, a_scales != nullptr);
    const hipError_t e = run_stream(p, pl, workspace, st);
    if (e != hipSuccess || pl.kg == 1) return e;
    return launch_proj_finish(static_cast<const float*>(workspace), pl.kg, 16 * pl.tb, out, p.M, p.M_out, p.N, 1, s, a_scales, w_scales, st);
}

}  // namespace shiftattn
