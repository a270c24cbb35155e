// Data-movement kernels of the path: send-side pack and receive-side unpack of the two SP
// all-to-alls (Algorithm 1), and the KV-cache append (Sec. 2.2).  All three are pure byte moves
// bound by HBM bandwidth: every thread moves whole 16-byte vectors, each workgroup issues four
// independent loads per thread before its stores, and consecutive lanes touch consecutive
// vectors of the output so that stores are fully coalesced and loads come in runs of at least one
// head vector (D * elem_size bytes).
#include "internal.h"

#include <type_traits>

namespace shiftattn {

namespace {

constexpr int kThreads = 256;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));  // one 8-byte vector
constexpr int kUnroll = 2;  // 16-byte vectors per thread: 2 measured best on the 512 MiB exchange (1: -2 %, 4: -3 %, 8: -40 %)

// One workgroup writes kThreads*kUnroll consecutive vectors of send[p].  The destination index is
// the fastest-varying part of the workgroup id, so the P workgroups that read the same input rows run
// together and the input is streamed once, front to back, while the P outputs advance in step.
__global__ __launch_bounds__(kThreads) void pack_seq2head_kernel(const u32x4* __restrict__ in,
                                                                 u32x4* __restrict__ out, XchgShape s,
                                                                 uint32_t row_vecs, uint32_t dest_vecs) {
    const int p = blockIdx.x % s.P;
    const uint32_t chunk = blockIdx.x / s.P;
    const int kv0 = s.h_kv ? static_cast<int>((static_cast<int64_t>(p) * s.h_kv) / s.P) : 0;
    const uint32_t in_row_heads = s.h + 2 * s.h_kv;
    const uint32_t first = chunk * (kThreads * kUnroll) + threadIdx.x;
    u32x4 v[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
        const uint32_t idx = first + k * kThreads;
        v[k] = u32x4{0u, 0u, 0u, 0u};
        if (idx < dest_vecs) {
            const uint32_t t = idx / row_vecs;
            const uint32_t c = idx - t * row_vecs;
            const uint32_t head = c / s.vec_per_head;
            const uint32_t dv = c - head * s.vec_per_head;
            uint32_t src_head;
            if (head < static_cast<uint32_t>(s.hq_l)) src_head = p * s.hq_l + head;
            else if (head < static_cast<uint32_t>(s.hq_l + s.hkv_l)) src_head = s.h + kv0 + (head - s.hq_l);
            else src_head = s.h + s.h_kv + kv0 + (head - s.hq_l - s.hkv_l);
            if (t < static_cast<uint32_t>(s.T))
                v[k] = __builtin_nontemporal_load(
                    in + (static_cast<size_t>(t) * in_row_heads + src_head) * s.vec_per_head + dv);
        }
    }
    u32x4* dst = out + static_cast<size_t>(p) * dest_vecs;
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
        const uint32_t idx = first + k * kThreads;
        if (idx < dest_vecs) __builtin_nontemporal_store(v[k], dst + idx);
    }
}

// One workgroup writes kThreads*kUnroll consecutive vectors of out[T][h][D].
__global__ __launch_bounds__(kThreads) void unpack_head2seq_kernel(const u32x4* __restrict__ in,
                                                                   u32x4* __restrict__ out, XchgShape s,
                                                                   uint32_t row_vecs, uint32_t out_vecs) {
    const uint32_t first = blockIdx.x * (kThreads * kUnroll) + threadIdx.x;
    u32x4 v[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
        const uint32_t idx = first + k * kThreads;
        if (idx < out_vecs) {
            const uint32_t t = idx / row_vecs;
            const uint32_t c = idx - t * row_vecs;
            const uint32_t head = c / s.vec_per_head;
            const uint32_t dv = c - head * s.vec_per_head;
            const uint32_t p = head / s.hq_l;
            const uint32_t j = head - p * s.hq_l;
            v[k] = __builtin_nontemporal_load(
                in + ((static_cast<size_t>(p) * s.T_pad + t) * s.hq_l + j) * s.vec_per_head + dv);
        }
    }
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) {
        const uint32_t idx = first + k * kThreads;
        if (idx < out_vecs) __builtin_nontemporal_store(v[k], out + idx);
    }
}

// One thread moves one 16-byte piece of a new K row and the matching piece of the V row.
// K keeps its row shape (one vector store); V is stored dimension-major inside the block, so its
// elements are scattered with a stride of one block row.
template <typename Elem>
__global__ __launch_bounds__(kThreads) void kv_write_kernel(const Elem* __restrict__ k_new,
                                                            const Elem* __restrict__ v_new,
                                                            const int64_t* __restrict__ slots, int n_tokens,
                                                            Elem* __restrict__ cache, int hkv_l, int D,
                                                            int64_t kv_stride) {
    constexpr int kPer = 16 / sizeof(Elem);
    const int vec_per_head = D / kPer;
    const int64_t id = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t total = static_cast<int64_t>(n_tokens) * hkv_l * vec_per_head;
    if (id >= total) return;
    const int dv = static_cast<int>(id % vec_per_head);
    const int g = static_cast<int>((id / vec_per_head) % hkv_l);
    const int64_t i = id / (static_cast<int64_t>(vec_per_head) * hkv_l);
    const int64_t slot = slots[i];
    if (slot < 0) return;
    const int64_t blk = slot / kBlockSize;
    const int off = static_cast<int>(slot % kBlockSize);
    const size_t src = static_cast<size_t>(i) * kv_stride + static_cast<size_t>(g) * D + dv * kPer;
    const u32x4 kvec = *reinterpret_cast<const u32x4*>(k_new + src);
    *reinterpret_cast<u32x4*>(cache + cache_part_offset(blk, g, 0, hkv_l, D) + static_cast<size_t>(off) * D +
                              dv * kPer) = kvec;
    union {
        u32x4 v;
        Elem e[kPer];
    } u;
    u.v = *reinterpret_cast<const u32x4*>(v_new + src);
    Elem* vdst = cache + cache_part_offset(blk, g, 1, hkv_l, D) + static_cast<size_t>(dv * kPer) * kBlockSize + off;
#pragma unroll
    for (int j = 0; j < kPer; ++j) vdst[j * kBlockSize] = u.e[j];
}

// bf16, D = 128.  A run is a stretch of consecutive new tokens whose slots are consecutive inside one
// cache block (at most 16 tokens).  Workgroup w looks at tokens 16 w .. 16 w + 15 and writes every run
// that *starts* there, to its end - up to 15 tokens into the next window, whose workgroup does not
// touch them.  So however the token index is aligned against the blocks (a batch of prefills of
// arbitrary lengths, a chunk that starts in the middle of a block), a full run fills its cache block
// with one pass: K rows as they come, V transposed through LDS and written as 4 KiB of consecutive
// bytes.  Short runs (first and last block of a sequence, single decode tokens, rows next to padding)
// write the part of each V row they own.  Every token belongs to exactly one run, so every cache
// element is written once and every input row read once; padding rows (negative slots) start no run.
// kFp8: the cache holds FP8 E4M3 codes (one byte per element) of x / scale instead of the bf16 values.
template <bool kFp8>
__global__ __launch_bounds__(kThreads) void kv_write_block_kernel(const uint16_t* __restrict__ k_new,
                                                                  const uint16_t* __restrict__ v_new,
                                                                  const int64_t* __restrict__ slots, int n_tokens,
                                                                  void* __restrict__ cache_v, int hkv_l,
                                                                  int64_t kv_stride, float k_scale, float v_scale) {
    using CE = typename std::conditional<kFp8, uint8_t, uint16_t>::type;    // cache element
    using Piece = typename std::conditional<kFp8, u32x2, u32x4>::type;       // eight cache elements
    constexpr int D = 128, kPitch = D + 16 / sizeof(CE);  // LDS row pitch in elements: 16-byte aligned, 4-bank skew per row
    __shared__ __attribute__((aligned(16))) CE tile[kBlockSize * kPitch];
    CE* cache = static_cast<CE*>(cache_v);
    const int g = blockIdx.y;
    const int lane16 = threadIdx.x & 15;
    const int64_t w0 = static_cast<int64_t>(blockIdx.x) * kBlockSize;
    // which tokens of the window start a run (every wavefront computes the same 16 bits)
    uint32_t starts;
    {
        const int64_t i = w0 + lane16;
        const int64_t s = i < n_tokens ? slots[i] : -1;
        const int64_t sp = i > 0 && i <= n_tokens ? slots[i - 1] : -2;
        const bool st = s >= 0 && ((s % kBlockSize) == 0 || sp != s - 1);
        starts = static_cast<uint32_t>(__builtin_amdgcn_ballot_w64(st)) & 0xFFFFu;
    }
    const int t_loc = threadIdx.x >> 4, dv = lane16;    // loader: token of the run, eight elements of its row
    const int d = threadIdx.x >> 1, h = threadIdx.x & 1;  // writer of V: head-dim row, half of its 16 positions
    auto encode = [&](u32x4 x, float scale) -> Piece {
        if constexpr (kFp8) {
            float f[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f[2 * j] = __uint_as_float(x[j] << 16);
                f[2 * j + 1] = __uint_as_float(x[j] & 0xFFFF0000u);
            }
            Piece r;
            r[0] = e4m3_pair(f[0], f[1], scale) | (e4m3_pair(f[2], f[3], scale) << 16);
            r[1] = e4m3_pair(f[4], f[5], scale) | (e4m3_pair(f[6], f[7], scale) << 16);
            return r;
        } else {
            return x;
        }
    };
    auto run_length = [&](int64_t i0, int64_t slot0) -> int {   // tokens from i0 on that continue slot0 inside its block
        const int64_t i = i0 + lane16;
        const bool cont = static_cast<int>(slot0 % kBlockSize) + lane16 < kBlockSize && i < n_tokens && slots[i] == slot0 + lane16;
        const uint32_t m = static_cast<uint32_t>(__builtin_amdgcn_ballot_w64(cont)) & 0xFFFFu;
        return __builtin_ctz(~m);
    };
    auto write_run = [&](int64_t i0, int64_t slot0, int len) {   // tokens i0 .. i0 + len - 1 into slots slot0 .. of one block
        const int off = static_cast<int>(slot0 % kBlockSize);
        const int64_t blk = slot0 / kBlockSize;
        if (t_loc < len) {
            const size_t src = static_cast<size_t>(i0 + t_loc) * kv_stride + static_cast<size_t>(g) * D + dv * 8;
            // rows and cache lines are touched once by this kernel: streaming loads and stores
            const u32x4 kvec = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(k_new + src));
            const u32x4 vvec = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(v_new + src));
            __builtin_nontemporal_store(encode(kvec, k_scale),
                                        reinterpret_cast<Piece*>(cache + cache_part_offset(blk, g, 0, hkv_l, D) +
                                                                 static_cast<size_t>(off + t_loc) * D + dv * 8));
            *reinterpret_cast<Piece*>(tile + t_loc * kPitch + dv * 8) = encode(vvec, v_scale);
        }
        __syncthreads();
        // positions 8 h .. 8 h + 7 of V row d; position p holds token p - off of the run
        CE* vrow = cache + cache_part_offset(blk, g, 1, hkv_l, D) + static_cast<size_t>(d) * kBlockSize + 8 * h;
        const int lo = max(off - 8 * h, 0), hi = min(off + len - 8 * h, 8);   // valid positions of this piece: [lo, hi)
        if (lo == 0 && hi == 8) {
            union {
                Piece v;
                CE e[8];
            } o;
#pragma unroll
            for (int j = 0; j < 8; ++j) o.e[j] = tile[(8 * h + j - off) * kPitch + d];
            __builtin_nontemporal_store(o.v, reinterpret_cast<Piece*>(vrow));
        } else {
            for (int j = lo; j < hi; ++j) vrow[j] = tile[(8 * h + j - off) * kPitch + d];
        }
    };
    if (__builtin_popcount(starts) <= 2) {   // the usual windows: inside a sequence, or across the end of one
        while (starts) {   // uniform
            const int t0 = __builtin_ctz(starts);
            starts &= starts - 1;
            const int64_t i0 = w0 + t0;
            const int64_t slot0 = slots[i0];
            write_run(i0, slot0, run_length(i0, slot0));
            if (starts) __syncthreads();   // the next run reuses the tile
        }
        return;
    }
    // Many short runs (decode tokens, rows between padding): every token of the window from the first start on belongs
    // to a run that starts here, so they are all loaded at once and scattered token by token; what the last run has
    // beyond the window follows as one run.
    __shared__ int64_t slot_s[kBlockSize];
    const int t_first = __builtin_ctz(starts), t_last = 31 - __builtin_clz(starts);
    {
        const int64_t i = w0 + t_loc;
        const int64_t slot = t_loc >= t_first && i < n_tokens ? slots[i] : -1;
        if (slot >= 0) {
            const size_t src = static_cast<size_t>(i) * kv_stride + static_cast<size_t>(g) * D + dv * 8;
            const u32x4 kvec = *reinterpret_cast<const u32x4*>(k_new + src);
            const u32x4 vvec = *reinterpret_cast<const u32x4*>(v_new + src);
            *reinterpret_cast<Piece*>(cache + cache_part_offset(slot / kBlockSize, g, 0, hkv_l, D) +
                                      static_cast<size_t>(slot % kBlockSize) * D + dv * 8) = encode(kvec, k_scale);
            *reinterpret_cast<Piece*>(tile + t_loc * kPitch + dv * 8) = encode(vvec, v_scale);
        }
        if (dv == 0) slot_s[t_loc] = slot;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 8; ++r) {   // lanes run over the tokens of a head-dim row first
        const int item = r * kThreads + threadIdx.x, dd = item >> 4, t = item & 15;
        const int64_t sl = slot_s[t];
        if (sl >= 0)
            cache[cache_part_offset(sl / kBlockSize, g, 1, hkv_l, D) + static_cast<size_t>(dd) * kBlockSize + sl % kBlockSize] = tile[t * kPitch + dd];
    }
    const int64_t i_last = w0 + t_last, slot_last = slots[i_last];
    const int beyond = t_last + run_length(i_last, slot_last) - kBlockSize;   // tokens of the last run past the window
    if (beyond > 0) {
        __syncthreads();
        write_run(w0 + kBlockSize, slot_last + (kBlockSize - t_last), beyond);
    }
}

// FP8 E4M3 cache: one thread quantises eight consecutive head-dim elements of one (token, KV head) for
// K and for V.  code = nearest E4M3 value of x / scale (float32 quotient, ties to the even code, clamped
// to +-448 first so that nothing overflows; a NaN quotient gives a NaN code).  K codes go out as one
// 8-byte store, V codes as eight byte stores into the dimension-major rows.
__device__ inline float elem_to_float(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }
__device__ inline float elem_to_float(float f) { return f; }


template <typename Elem>
__global__ __launch_bounds__(kThreads) void kv_write_fp8_kernel(const Elem* __restrict__ k_new,
                                                                const Elem* __restrict__ v_new,
                                                                const int64_t* __restrict__ slots, int n_tokens,
                                                                uint8_t* __restrict__ cache, int hkv_l, int D,
                                                                int64_t kv_stride, float k_scale, float v_scale) {
    const int groups = D / 8;
    const int64_t id = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (id >= static_cast<int64_t>(n_tokens) * hkv_l * groups) return;
    const int dg = static_cast<int>(id % groups);
    const int g = static_cast<int>((id / groups) % hkv_l);
    const int64_t i = id / (static_cast<int64_t>(groups) * hkv_l);
    const int64_t slot = slots[i];
    if (slot < 0) return;
    const int64_t blk = slot / kBlockSize;
    const int off = static_cast<int>(slot % kBlockSize);
    const size_t src = static_cast<size_t>(i) * kv_stride + static_cast<size_t>(g) * D + dg * 8;
    float kx[8], vx[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        kx[j] = elem_to_float(k_new[src + j]);
        vx[j] = elem_to_float(v_new[src + j]);
    }
    uint32_t kc[2], vc[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        kc[h] = e4m3_pair(kx[4 * h], kx[4 * h + 1], k_scale) | (e4m3_pair(kx[4 * h + 2], kx[4 * h + 3], k_scale) << 16);
        vc[h] = e4m3_pair(vx[4 * h], vx[4 * h + 1], v_scale) | (e4m3_pair(vx[4 * h + 2], vx[4 * h + 3], v_scale) << 16);
    }
    uint8_t* kdst = cache + cache_part_offset(blk, g, 0, hkv_l, D) + static_cast<size_t>(off) * D + dg * 8;
    *reinterpret_cast<u32x2*>(kdst) = u32x2{kc[0], kc[1]};
    uint8_t* vdst = cache + cache_part_offset(blk, g, 1, hkv_l, D) + static_cast<size_t>(dg * 8) * kBlockSize + off;
#pragma unroll
    for (int j = 0; j < 8; ++j) vdst[j * kBlockSize] = static_cast<uint8_t>(vc[j >> 2] >> (8 * (j & 3)));
}

// FP8 E4M3 cache blocks of the contexts of a batch, widened to bf16 (D = 128): one workgroup per
// (sequence, block index, KV head), one 16-byte piece of codes per thread.  K and V^T keep their
// arrangement, so element e of the 4 KiB of codes becomes element e of the 8 KiB of bf16.
__global__ __launch_bounds__(kThreads) void fp8_blocks_to_bf16_kernel(const uint8_t* __restrict__ cache,
                                                                      const int32_t* __restrict__ block_table,
                                                                      int max_blocks, const int32_t* __restrict__ seq_lens,
                                                                      int nb, int hkv_l, uint16_t* __restrict__ scratch,
                                                                      int32_t* __restrict__ table_out) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const int i = blockIdx.x % nb, s = blockIdx.x / nb, g = blockIdx.y;
    const int dst_blk = s * nb + i;
    if (g == 0 && threadIdx.x == 0) table_out[dst_blk] = dst_blk;
    if (i * kBlockSize >= seq_lens[s]) return;  // uniform: no token of the context in this block
    const int64_t src_blk = block_table[static_cast<size_t>(s) * max_blocks + i];
    constexpr int D = 128, kCodes = 2 * kBlockSize * D;  // codes (and bf16 elements) per (block, head)
    const u32x4 codes = *(reinterpret_cast<const u32x4*>(cache + (static_cast<size_t>(src_blk) * hkv_l + g) * kCodes) + threadIdx.x);
    u32x4 lo, hi;
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        lo[2 * w] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(codes[w]), 1.0f, false));
        lo[2 * w + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(codes[w]), 1.0f, true));
        hi[2 * w] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(codes[2 + w]), 1.0f, false));
        hi[2 * w + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(codes[2 + w]), 1.0f, true));
    }
    u32x4* dst = reinterpret_cast<u32x4*>(scratch + (static_cast<size_t>(dst_blk) * hkv_l + g) * kCodes) + 2 * threadIdx.x;
    dst[0] = lo;
    dst[1] = hi;
}

}  // namespace

hipError_t launch_fp8_blocks_to_bf16(const void* cache_fp8, const int32_t* block_table, int max_blocks,
                                     const int32_t* seq_lens, int num_seqs, int nb, int hkv_l, void* scratch_bf16,
                                     int32_t* table_out, hipStream_t st) {
    const int64_t wgs = static_cast<int64_t>(num_seqs) * nb;
    if (wgs == 0) return hipSuccess;
    if (wgs > 0x7FFFFFFF || hkv_l > 65535) return hipErrorInvalidValue;
    dim3 grid(static_cast<unsigned>(wgs), static_cast<unsigned>(hkv_l));
    fp8_blocks_to_bf16_kernel<<<grid, kThreads, 0, st>>>(static_cast<const uint8_t*>(cache_fp8), block_table, max_blocks,
                                                         seq_lens, nb, hkv_l, static_cast<uint16_t*>(scratch_bf16), table_out);
    return hipGetLastError();
}

hipError_t launch_pack(const void* qkv, void* send, const XchgShape& s, hipStream_t st) {
    const uint32_t row_vecs = static_cast<uint32_t>(s.hq_l + 2 * s.hkv_l) * s.vec_per_head;
    const uint32_t dest_vecs = static_cast<uint32_t>(s.T_pad) * row_vecs;
    if (dest_vecs == 0) return hipSuccess;
    const uint64_t chunks = (dest_vecs + kThreads * kUnroll - 1) / (kThreads * kUnroll);
    const unsigned grid = static_cast<unsigned>(chunks * s.P);  // < 2^31: dest_vecs * P is bounded by the caller
    pack_seq2head_kernel<<<grid, kThreads, 0, st>>>(static_cast<const u32x4*>(qkv), static_cast<u32x4*>(send), s,
                                                    row_vecs, dest_vecs);
    return hipGetLastError();
}

hipError_t launch_unpack(const void* recv, void* out, const XchgShape& s, hipStream_t st) {
    const uint32_t row_vecs = static_cast<uint32_t>(s.h) * s.vec_per_head;
    const uint32_t out_vecs = static_cast<uint32_t>(s.T) * row_vecs;
    if (out_vecs == 0) return hipSuccess;
    dim3 grid((out_vecs + kThreads * kUnroll - 1) / (kThreads * kUnroll));
    unpack_head2seq_kernel<<<grid, kThreads, 0, st>>>(static_cast<const u32x4*>(recv), static_cast<u32x4*>(out), s,
                                                      row_vecs, out_vecs);
    return hipGetLastError();
}

// Rows of bf16 values as FP8 E4M3 codes with one scale per row: scale = max |x| / 448 (float32 quotient; 1 for a row
// of zeros), code = e4m3(x / scale).  One workgroup per row; a thread keeps up to kQuantPieces 16-byte pieces of the
// row in registers between the maximum and the conversion, longer rows are read a second time.
constexpr int kQuantPieces = 8;
__global__ __launch_bounds__(kThreads) void quantize_rows_fp8_kernel(const uint16_t* __restrict__ x, uint8_t* __restrict__ codes,
                                                                     float* __restrict__ scales, int cols, int seg_len,
                                                                     int64_t seg_stride, int64_t row_stride) {
    __shared__ float wave_max[kThreads / 64];
    const int64_t row = blockIdx.x;
    const int pieces = cols / 8;
    auto offset = [&](int piece) -> size_t {
        const int k = piece * 8, seg = k / seg_len;
        return static_cast<size_t>(seg) * seg_stride + static_cast<size_t>(row) * row_stride + (k - seg * seg_len);
    };
    u32x4 held[kQuantPieces];
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < kQuantPieces; ++i) {
        const int piece = threadIdx.x + i * kThreads;
        held[i] = u32x4{0u, 0u, 0u, 0u};
        if (piece < pieces) held[i] = *reinterpret_cast<const u32x4*>(x + offset(piece));
#pragma unroll
        for (int j = 0; j < 4; ++j)
            amax = fmaxf(amax, fmaxf(fabsf(__uint_as_float(held[i][j] << 16)), fabsf(__uint_as_float(held[i][j] & 0xFFFF0000u))));
    }
    for (int piece = threadIdx.x + kQuantPieces * kThreads; piece < pieces; piece += kThreads) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(x + offset(piece));
#pragma unroll
        for (int j = 0; j < 4; ++j)
            amax = fmaxf(amax, fmaxf(fabsf(__uint_as_float(v[j] << 16)), fabsf(__uint_as_float(v[j] & 0xFFFF0000u))));
    }
    // fmaxf drops NaN operands: a row with NaN elements is scaled by its largest number, the NaNs become NaN codes
#pragma unroll
    for (int sh = 32; sh > 0; sh >>= 1) amax = fmaxf(amax, __shfl_xor(amax, sh));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
    const float scale = amax > 0.f ? amax / 448.f : 1.f;
    if (threadIdx.x == 0) scales[row] = scale;
    auto encode = [&](u32x4 v) -> u32x2 {
        float f[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[2 * j] = __uint_as_float(v[j] << 16);
            f[2 * j + 1] = __uint_as_float(v[j] & 0xFFFF0000u);
        }
        return u32x2{e4m3_pair(f[0], f[1], scale) | (e4m3_pair(f[2], f[3], scale) << 16),
                     e4m3_pair(f[4], f[5], scale) | (e4m3_pair(f[6], f[7], scale) << 16)};
    };
#pragma unroll
    for (int i = 0; i < kQuantPieces; ++i) {
        const int piece = threadIdx.x + i * kThreads;
        if (piece < pieces) *reinterpret_cast<u32x2*>(codes + offset(piece)) = encode(held[i]);
    }
    for (int piece = threadIdx.x + kQuantPieces * kThreads; piece < pieces; piece += kThreads)
        *reinterpret_cast<u32x2*>(codes + offset(piece)) = encode(*reinterpret_cast<const u32x4*>(x + offset(piece)));
}

hipError_t launch_quantize_rows_fp8(const void* x, void* codes, float* scales, int rows, int cols, int seg_len,
                                    int64_t seg_stride, int64_t row_stride, hipStream_t st) {
    if (rows == 0) return hipSuccess;
    quantize_rows_fp8_kernel<<<static_cast<unsigned>(rows), kThreads, 0, st>>>(static_cast<const uint16_t*>(x),
                                                                               static_cast<uint8_t*>(codes), scales, cols, seg_len,
                                                                               seg_stride, row_stride);
    return hipGetLastError();
}

hipError_t launch_kv_write(const void* k_new, const void* v_new, const int64_t* slots, int n_tokens, void* cache,
                           const AttnShape& a, hipStream_t st) {
    if (a.kv_fp8()) {
        const int64_t items = static_cast<int64_t>(n_tokens) * a.hkv_l * (a.D / 8);
        if (items == 0) return hipSuccess;
        const unsigned grid8 = static_cast<unsigned>((items + kThreads - 1) / kThreads);
        if (a.elem == 2 && a.D == 128 && a.hkv_l <= 65535) {
            dim3 g2(static_cast<unsigned>((n_tokens + kBlockSize - 1) / kBlockSize), static_cast<unsigned>(a.hkv_l));
            kv_write_block_kernel<true><<<g2, kThreads, 0, st>>>(static_cast<const uint16_t*>(k_new),
                                                                 static_cast<const uint16_t*>(v_new), slots, n_tokens, cache,
                                                                 a.hkv_l, a.kv_stride, a.k_scale, a.v_scale);
        } else if (a.elem == 2)
            kv_write_fp8_kernel<uint16_t><<<grid8, kThreads, 0, st>>>(
                static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new), slots, n_tokens,
                static_cast<uint8_t*>(cache), a.hkv_l, a.D, a.kv_stride, a.k_scale, a.v_scale);
        else
            kv_write_fp8_kernel<float><<<grid8, kThreads, 0, st>>>(
                static_cast<const float*>(k_new), static_cast<const float*>(v_new), slots, n_tokens,
                static_cast<uint8_t*>(cache), a.hkv_l, a.D, a.kv_stride, a.k_scale, a.v_scale);
        return hipGetLastError();
    }
    const int64_t total = static_cast<int64_t>(n_tokens) * a.hkv_l * (a.D * a.elem / 16);
    if (total == 0) return hipSuccess;
    const unsigned grid = static_cast<unsigned>((total + kThreads - 1) / kThreads);
    if (a.elem == 2 && a.D == 128 && a.hkv_l <= 65535) {
        dim3 g2(static_cast<unsigned>((n_tokens + kBlockSize - 1) / kBlockSize), static_cast<unsigned>(a.hkv_l));
        kv_write_block_kernel<false><<<g2, kThreads, 0, st>>>(static_cast<const uint16_t*>(k_new),
                                                              static_cast<const uint16_t*>(v_new), slots, n_tokens, cache,
                                                              a.hkv_l, a.kv_stride, 1.f, 1.f);
        return hipGetLastError();
    }
    if (a.elem == 2)
        kv_write_kernel<uint16_t><<<grid, kThreads, 0, st>>>(static_cast<const uint16_t*>(k_new),
                                                            static_cast<const uint16_t*>(v_new), slots, n_tokens,
                                                            static_cast<uint16_t*>(cache), a.hkv_l, a.D, a.kv_stride);
    else
        kv_write_kernel<uint32_t><<<grid, kThreads, 0, st>>>(static_cast<const uint32_t*>(k_new),
                                                            static_cast<const uint32_t*>(v_new), slots, n_tokens,
                                                            static_cast<uint32_t*>(cache), a.hkv_l, a.D, a.kv_stride);
    return hipGetLastError();
}

}  // namespace shiftattn
