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
// Kernel: 256 x 256 output tile per workgroup, K in steps of 64, eight wavefronts (4 along the features
// x 2 along the tokens), v_mfma_f32_32x32x16_bf16 with the weight rows as A operand and the token rows
// as B operand, so a lane ends up with runs of four consecutive features of one token (8-byte stores).
// Both tiles of a step (2 x 32 KiB) arrive by direct-to-LDS loads, double buffered; a row of 64 k (128
// bytes) keeps its eight 16-byte pieces at positions piece ^ ((row / 2) % 8), which makes the operand
// reads (32 consecutive rows, one piece column) conflict-free.
#include "internal.h"

namespace shiftattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTile = 256;                 // rows of either operand per workgroup
constexpr int kBK = 64;                    // k per step
constexpr int kRowBytes = kBK * 2;         // 128
constexpr int kOperandBytes = kTile * kRowBytes;   // 32768
constexpr int kStage = 2 * kOperandBytes;  // weights, then tokens
constexpr int kGemmLds = 2 * kStage;       // 131072
constexpr int kGemmThreads = 512;
constexpr int kHeadDim = 128;

__device__ inline bf16x8 frag(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct GemmParams {
    const uint16_t* __restrict__ w;   // [N][K]
    const uint16_t* __restrict__ x;   // token rows; see mode
    uint16_t* __restrict__ c;
    int M, M_out, N, K;               // M token rows exist, rows M..M_out-1 of the result are written as zeros
    // mode 0 (qkv_proj_pack): x dense [M][K]; result columns scattered to send buffers (XchgShape below)
    // mode 1 (unpack_o_proj): x gathered from recv [P][T_pad][hq_l][128] (k = (p hq_l + j) 128 + e); result dense [M][N]
    int mode;
    XchgShape s;
};

__global__ __launch_bounds__(kGemmThreads, 2) void proj_gemm_kernel(GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    typedef __attribute__((address_space(3))) void* lds_ptr;
    typedef const __attribute__((address_space(1))) void* glb_ptr;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int l32 = lane & 31, half = lane >> 5;
    const int wn = wave & 3, wm = wave >> 2;
    // feature tiles vary fastest: workgroups that run together share the token rows in L2
    const int n_tiles = p.N / kTile;
    const int n0 = (blockIdx.x % n_tiles) * kTile, m0 = (blockIdx.x / n_tiles) * kTile;

    // ---- direct-to-LDS loads: this wavefront fills rows 32 wave .. 32 wave + 31 of both operand tiles, eight rows
    // (1 KiB) per instruction; lane -> row 8 j + lane / 8, LDS piece position lane % 8, logical piece = position ^ key
    const int ld_row = lane >> 3, ld_pos = lane & 7;
    size_t w_src[4], x_src[4];   // element offsets of this lane's piece at k = 0
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 32 * wave + 8 * j + ld_row;
        const int piece = ld_pos ^ ((row >> 1) & 7);
        w_src[j] = static_cast<size_t>(n0 + row) * p.K + piece * 8;
        const int m = min(m0 + row, p.M - 1);   // rows past the end re-read the last one; they are not stored
        x_src[j] = p.mode == 0 ? static_cast<size_t>(m) * p.K + piece * 8
                               : static_cast<size_t>(m) * p.s.hq_l * kHeadDim + piece * 8;
    }
    auto x_k_off = [&](int k0) -> size_t {   // where k-tile k0 of a token row starts (wavefront-uniform)
        if (p.mode == 0) return static_cast<size_t>(k0);
        const int head = k0 / kHeadDim, pp = head / p.s.hq_l, j = head - pp * p.s.hq_l;
        return (static_cast<size_t>(pp) * p.s.T_pad * p.s.hq_l + j) * kHeadDim + (k0 % kHeadDim);
    };
    auto load_stage = [&](int k0, int stage) {
        unsigned char* dst = lds + stage * kStage + (32 * wave) * kRowBytes;
        const size_t xo = x_k_off(k0);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            __builtin_amdgcn_global_load_lds((glb_ptr)(p.w + w_src[j] + k0), (lds_ptr)(dst + j * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            __builtin_amdgcn_global_load_lds((glb_ptr)(p.x + x_src[j] + xo), (lds_ptr)(dst + kOperandBytes + j * 1024), 16, 0, 0);
    };

    // ---- operand reads: row l32 of a 32-row tile, piece 2 ks + half
    const int key = (l32 >> 1) & 7;   // 32-row tiles start at multiples of 32: the key depends on l32 only
    int rd[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) rd[ks] = l32 * kRowBytes + (((2 * ks + half) ^ key) << 4);
    const int a_base = (wn * 64) * kRowBytes;                    // weight rows of this wavefront
    const int b_base = kOperandBytes + (wm * 128) * kRowBytes;   // token rows of this wavefront

    f32x16 acc[2][4];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nt][mt][r] = 0.f;

    const int k_steps = p.K / kBK;
    load_stage(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();
    for (int kt = 0; kt < k_steps; ++kt) {
        const int st = kt & 1;
        if (kt + 1 < k_steps) load_stage((kt + 1) * kBK, st ^ 1);
        const unsigned char* base = lds + st * kStage;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 a[2], b[4];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) a[nt] = *reinterpret_cast<const u32x4*>(base + a_base + nt * 32 * kRowBytes + rd[ks]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) b[mt] = *reinterpret_cast<const u32x4*>(base + b_base + mt * 32 * kRowBytes + rd[ks]);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
                    acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(a[nt]), frag(b[mt]), acc[nt][mt], 0, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
    }

    // ---- result: register r of acc[nt][mt] is feature 32 nt + 8 (r / 4) + 4 half + r % 4 of token 32 mt + l32
    const int f_wave = n0 + wn * 64;           // first feature of this wavefront; its 64 features lie in one head
    auto store_rows = [&](uint16_t* dst_row0, size_t row_stride) {   // dst_row0: feature f_wave of token row 0
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            const int m = m0 + wm * 128 + mt * 32 + l32;
            if (m >= p.M_out) continue;
            uint16_t* row = dst_row0 + static_cast<size_t>(m) * row_stride + 4 * half;
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    bf16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(m < p.M ? acc[nt][mt][4 * r4 + e] : 0.f);
                    *reinterpret_cast<u32x2*>(row + 32 * nt + 8 * r4) = __builtin_bit_cast(u32x2, v);
                }
        }
    };
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

hipError_t launch(const GemmParams& p, hipStream_t st) {
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&proj_gemm_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const int64_t wgs = static_cast<int64_t>(p.N / kTile) * ((p.M_out + kTile - 1) / kTile);
    if (wgs == 0) return hipSuccess;
    if (wgs > 0x7FFFFFFF) return hipErrorInvalidValue;
    proj_gemm_kernel<<<static_cast<unsigned>(wgs), kGemmThreads, kGemmLds, st>>>(p);
    return hipGetLastError();
}

}  // namespace

// bf16, head_dim 128; the feature dimension of either product must be a multiple of the 256-wide tile
bool qkv_proj_pack_supported(const XchgShape& s, int d_model, int elem) {
    return elem == 2 && s.vec_per_head * 8 == kHeadDim && d_model > 0 && d_model % kBK == 0 && (s.h + 2 * s.h_kv) % 2 == 0;
}
bool unpack_o_proj_supported(const XchgShape& s, int d_model, int elem) {
    return elem == 2 && s.vec_per_head * 8 == kHeadDim && d_model > 0 && d_model % kTile == 0 && s.h > 0;
}

hipError_t launch_qkv_proj_pack(const void* x, const void* w_qkv, void* send, int d_model, const XchgShape& s, hipStream_t st) {
    GemmParams p;
    p.w = static_cast<const uint16_t*>(w_qkv);
    p.x = static_cast<const uint16_t*>(x);
    p.c = static_cast<uint16_t*>(send);
    p.M = s.T;
    p.M_out = s.T_pad;
    p.N = (s.h + 2 * s.h_kv) * kHeadDim;
    p.K = d_model;
    p.mode = 0;
    p.s = s;
    if (s.T == 0) return launch_pack(nullptr, send, s, st);  // only padding rows: the pack kernel writes the zeros
    return launch(p, st);
}

hipError_t launch_unpack_o_proj(const void* recv, const void* w_o, void* out, int d_model, const XchgShape& s, hipStream_t st) {
    GemmParams p;
    p.w = static_cast<const uint16_t*>(w_o);
    p.x = static_cast<const uint16_t*>(recv);
    p.c = static_cast<uint16_t*>(out);
    p.M = s.T;
    p.M_out = s.T;
    p.N = d_model;
    p.K = s.h * kHeadDim;
    p.mode = 1;
    p.s = s;
    if (s.T == 0) return hipSuccess;
    return launch(p, st);
}

}  // namespace shiftattn
