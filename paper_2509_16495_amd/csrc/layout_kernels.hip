// Data-movement kernels of the path: send-side pack and receive-side unpack of the two SP
// all-to-alls (Algorithm 1), and the KV-cache append (Sec. 2.2).  All three are pure byte moves
// bound by HBM bandwidth: every thread moves whole 16-byte vectors, each workgroup issues four
// independent loads per thread before its stores, and consecutive lanes touch consecutive
// vectors of the output so that stores are fully coalesced and loads come in runs of at least one
// head vector (D * elem_size bytes).
#include "internal.h"

namespace shiftattn {

namespace {

constexpr int kThreads = 256;
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

// bf16, D = 128: one workgroup appends 16 consecutive new tokens of one KV head.  When those tokens
// fill exactly one cache block in order (the usual case for a prefill chunk) the V rows are
// transposed through LDS and the block's V part is written as 4 KiB of consecutive bytes; any other
// slot pattern is scattered element by element out of the same LDS tile.  Same bytes in the cache either way.
__global__ __launch_bounds__(kThreads) void kv_write_block_kernel(const uint16_t* __restrict__ k_new,
                                                                  const uint16_t* __restrict__ v_new,
                                                                  const int64_t* __restrict__ slots, int n_tokens,
                                                                  uint16_t* __restrict__ cache, int hkv_l,
                                                                  int64_t kv_stride) {
    constexpr int D = 128, kPitch = D + 8;  // LDS row pitch in elements: 16-byte aligned, 4-bank skew per row
    __shared__ __attribute__((aligned(16))) uint16_t tile[kBlockSize * kPitch];
    __shared__ int64_t slot_s[kBlockSize];
    const int g = blockIdx.y;
    const int t_loc = threadIdx.x >> 4, dv = threadIdx.x & 15;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlockSize + t_loc;
    const bool in_range = i < n_tokens;
    // the rows are requested together with the slots (rows of padding tokens exist too, they are just not
    // written): one round trip to memory instead of two dependent ones
    u32x4 kvec = {0u, 0u, 0u, 0u}, vvec = {0u, 0u, 0u, 0u};
    if (in_range) {
        const size_t src = static_cast<size_t>(i) * kv_stride + static_cast<size_t>(g) * D + dv * 8;
        kvec = *reinterpret_cast<const u32x4*>(k_new + src);
        vvec = *reinterpret_cast<const u32x4*>(v_new + src);
    }
    const int64_t slot = in_range ? slots[i] : -1;
    const int64_t first = slots[static_cast<int64_t>(blockIdx.x) * kBlockSize];  // blockIdx.x * 16 < n_tokens
    const bool ordered = in_range && first >= 0 && (first % kBlockSize) == 0 && slot == first + t_loc;
    const bool whole_block = __syncthreads_and(ordered);
    if (in_range && slot >= 0) {
        const int64_t blk = slot / kBlockSize;
        const int off = static_cast<int>(slot % kBlockSize);
        *reinterpret_cast<u32x4*>(cache + cache_part_offset(blk, g, 0, hkv_l, D) + static_cast<size_t>(off) * D + dv * 8) = kvec;
    }
    *reinterpret_cast<u32x4*>(tile + t_loc * kPitch + dv * 8) = vvec;
    if (dv == 0) slot_s[t_loc] = slot;
    __syncthreads();
    if (!whole_block) {  // uniform
        // Any other slot pattern (a run that straddles two blocks, padding rows, the tail of the batch): element by
        // element out of the LDS tile, lanes running over the tokens of a head-dim row first, so that tokens that
        // are neighbours in a block leave as neighbouring 2-byte stores of one instruction.
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int item = r * kThreads + threadIdx.x, d = item >> 4, t = item & 15;
            const int64_t sl = slot_s[t];
            if (sl >= 0)
                cache[cache_part_offset(sl / kBlockSize, g, 1, hkv_l, D) + static_cast<size_t>(d) * kBlockSize + sl % kBlockSize] =
                    tile[t * kPitch + d];
        }
        return;
    }
    // thread -> (head-dim row d, half h): eight consecutive tokens of row d
    const int d = threadIdx.x >> 1, h = threadIdx.x & 1;
    union {
        u32x4 v;
        uint16_t e[8];
    } o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o.e[j] = tile[(8 * h + j) * kPitch + d];
    uint16_t* vblk = cache + cache_part_offset(first / kBlockSize, g, 1, hkv_l, D);
    *reinterpret_cast<u32x4*>(vblk + static_cast<size_t>(d) * kBlockSize + 8 * h) = o.v;
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
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    *reinterpret_cast<u32x2_t*>(kdst) = u32x2_t{kc[0], kc[1]};
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

hipError_t launch_kv_write(const void* k_new, const void* v_new, const int64_t* slots, int n_tokens, void* cache,
                           const AttnShape& a, hipStream_t st) {
    if (a.kv_fp8()) {
        const int64_t items = static_cast<int64_t>(n_tokens) * a.hkv_l * (a.D / 8);
        if (items == 0) return hipSuccess;
        const unsigned grid8 = static_cast<unsigned>((items + kThreads - 1) / kThreads);
        if (a.elem == 2)
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
        kv_write_block_kernel<<<g2, kThreads, 0, st>>>(static_cast<const uint16_t*>(k_new),
                                                       static_cast<const uint16_t*>(v_new), slots, n_tokens,
                                                       static_cast<uint16_t*>(cache), a.hkv_l, a.kv_stride);
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
