// General attention kernel and the merge of split-context partial results.
//
// attn_rows_kernel covers every element type, head_dim (multiple of 8, <= 256) and GQA ratio the
// boundary accepts, for prefill chunks and decode rows alike: one wavefront per (token, query head)
// row, lanes spread over 64 keys for q.k, then over the head dimension for p.V, online softmax in
// fp32 (Algorithm 1, boxed attention line; Sec. 2.2).  It is the reference-grade path for shapes
// the MFMA kernels do not take (fp32 tensors, head_dim != 128) and is not tuned for speed.
#include "internal.h"

namespace shiftattn {

namespace {

__device__ inline float to_float(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }
__device__ inline float to_float(float f) { return f; }
// value of an FP8 E4M3 code (the scale is applied by the caller)
__device__ inline float to_float(uint8_t c) { return __builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(c), false)[0]; }

__device__ inline uint16_t bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if (f != f) return 0x7FC0;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}
__device__ inline void store_elem(uint16_t* p, float f) { *p = bf16_rne(f); }
__device__ inline void store_elem(float* p, float f) { *p = f; }

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

constexpr int kWaves = 4;
constexpr int kMaxD = 256;

template <typename Elem, typename KvElem>
__global__ __launch_bounds__(kWaves * 64) void attn_rows_kernel(
    const Elem* __restrict__ q, const KvElem* __restrict__ cache, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ cu_seqlens_q, const int32_t* __restrict__ seq_lens, int num_seqs, int total_q,
    Elem* __restrict__ out, AttnShape a) {
    constexpr int kPer = 16 / sizeof(KvElem);  // cache elements per 16-byte vector
    __shared__ float q_s[kWaves][kMaxD];
    __shared__ float p_s[kWaves][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * kWaves + wave;
    if (row >= static_cast<int64_t>(total_q) * a.hq_l) return;  // whole wavefront leaves together
    const int tok = static_cast<int>(row / a.hq_l);
    const int j = static_cast<int>(row % a.hq_l);
    const int g = j / (a.hq_l / a.hkv_l);

    int s, pos;
    if (cu_seqlens_q == nullptr) {
        s = tok;
        pos = seq_lens[s] - 1;
    } else {
        int lo = 0, hi = num_seqs;  // last s with cu[s] <= tok
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (cu_seqlens_q[mid] <= tok) lo = mid; else hi = mid;
        }
        s = lo;
        const int q_len = cu_seqlens_q[s + 1] - cu_seqlens_q[s];
        pos = seq_lens[s] - q_len + (tok - cu_seqlens_q[s]);
    }
    const int32_t* table = block_table + static_cast<size_t>(s) * a.max_blocks;
    const int D = a.D;

    const Elem* q_row = q + static_cast<size_t>(tok) * a.q_stride + static_cast<size_t>(j) * D;
    for (int d = lane; d < D; d += 64) q_s[wave][d] = to_float(q_row[d]);
    __builtin_amdgcn_wave_barrier();

    float m_run = -INFINITY, l_run = 0.f;
    float o[kMaxD / 64] = {0.f, 0.f, 0.f, 0.f};

    for (int t0 = 0; t0 <= pos; t0 += 64) {
        const int t = t0 + lane;
        float logit = -INFINITY;
        if (t <= pos) {
            const int64_t blk = table[t / kBlockSize];
            const KvElem* k_row = cache + cache_part_offset(blk, g, 0, a.hkv_l, D) + static_cast<size_t>(t % kBlockSize) * D;
            float dot = 0.f;
            for (int dv = 0; dv < D / kPer; ++dv) {
                union { u32x4 v; KvElem e[kPer]; } u;
                u.v = *reinterpret_cast<const u32x4*>(k_row + dv * kPer);
#pragma unroll
                for (int x = 0; x < kPer; ++x) dot = fmaf(q_s[wave][dv * kPer + x], to_float(u.e[x]), dot);
            }
            logit = dot * (a.scale * a.k_scale);
        }
        const float m_new = fmaxf(m_run, wave_max(logit));  // finite: key t0 is always visible
        const float p = (t <= pos) ? expf(logit - m_new) : 0.f;
        const float alpha = expf(m_run - m_new);             // exp(-inf) = 0 on the first chunk
        l_run = l_run * alpha + wave_sum(p);
        m_run = m_new;
        p_s[wave][lane] = p;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int x = 0; x < kMaxD / 64; ++x) o[x] *= alpha;
        for (int b = 0; b < 4 && t0 + b * kBlockSize <= pos; ++b) {
            const int64_t blk = table[(t0 + b * kBlockSize) / kBlockSize];
            const KvElem* v_part = cache + cache_part_offset(blk, g, 1, a.hkv_l, D);
#pragma unroll
            for (int x = 0; x < kMaxD / 64; ++x) {
                const int d = lane + 64 * x;
                if (d < D) {
                    const KvElem* v_row = v_part + static_cast<size_t>(d) * kBlockSize;
#pragma unroll
                    for (int vv = 0; vv < kBlockSize / kPer; ++vv) {
                        union { u32x4 v; KvElem e[kPer]; } u;
                        u.v = *reinterpret_cast<const u32x4*>(v_row + vv * kPer);
#pragma unroll
                        for (int y = 0; y < kPer; ++y) {
                            const int off = vv * kPer + y;
                            // slots past the context may hold anything (also NaN): select, do not multiply
                            const float val = (t0 + b * kBlockSize + off <= pos) ? to_float(u.e[y]) : 0.f;
                            o[x] = fmaf(p_s[wave][b * kBlockSize + off], val, o[x]);
                        }
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    Elem* o_row = out + static_cast<size_t>(tok) * a.out_stride + static_cast<size_t>(j) * D;
    const float inv = l_run > 0.f ? a.v_scale / l_run : 0.f;  // a row without visible keys (padding) is zero
#pragma unroll
    for (int x = 0; x < kMaxD / 64; ++x) {
        const int d = lane + 64 * x;
        if (d < D) store_elem(o_row + d, o[x] * inv);
    }
}

// One workgroup per output row (token, head).  The row's (max, sum) pairs are fetched in parallel
// and turned into weights in LDS; then every thread owns head-dim elements and sums the weighted
// partials in part order with independent loads.
constexpr int kCombineThreads = 128;
constexpr int kCombineMaxParts = kMaxParts;

template <typename Elem>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(const float* __restrict__ o_part,
                                                                  const float* __restrict__ ml_part, int n_rows,
                                                                  int hq_l, int D, int n_parts, int mode,
                                                                  const int32_t* __restrict__ seq_lens, int chunk,
                                                                  Elem* __restrict__ out, int64_t out_stride,
                                                                  float out_scale) {
    __shared__ float w_s[kCombineMaxParts];
    __shared__ float l_s[kCombineMaxParts];
    __shared__ float red_s[kCombineThreads / 64];
    const int row = blockIdx.x;  // token * hq_l + head
    const int tok = row / hq_l, head = row % hq_l;
    int np = n_parts;
    if (mode == 1) np = (seq_lens[tok] + chunk - 1) / chunk;
    // partial row of part c: row0 + c * part_rows
    const size_t part_rows = static_cast<size_t>(n_rows) * hq_l;
    const size_t row0 = row;
    np = min(np, kCombineMaxParts);
    const int tid = threadIdx.x;
    // the first parts of this thread's output elements are requested before the weights are known,
    // so their latency overlaps that of the (max, sum) pairs
    constexpr int kEarly = 8;
    float early[kEarly];
    const int d0 = tid;  // D <= kCombineThreads * ceil: the common D = 128 gives one element per thread
    if (d0 < D) {
#pragma unroll
        for (int c = 0; c < kEarly; ++c) early[c] = c < np ? o_part[(row0 + c * part_rows) * D + d0] : 0.f;
    }
    float m_loc = -INFINITY;
    for (int c = tid; c < np; c += kCombineThreads) {
        const float m_c = ml_part[(c * part_rows + row0) * 2];
        w_s[c] = m_c;
        l_s[c] = ml_part[(c * part_rows + row0) * 2 + 1];
        m_loc = fmaxf(m_loc, m_c);
    }
    m_loc = wave_max(m_loc);
    if ((tid & 63) == 0) red_s[tid >> 6] = m_loc;
    __syncthreads();
    float m_star = red_s[0];
#pragma unroll
    for (int w = 1; w < kCombineThreads / 64; ++w) m_star = fmaxf(m_star, red_s[w]);
    for (int c = tid; c < np; c += kCombineThreads) {
        const float m_c = w_s[c];  // each slot is read and rewritten by the same thread
        w_s[c] = (m_c == -INFINITY) ? 0.f : exp2f(m_c - m_star);
    }
    __syncthreads();
    float l_star = 0.f;  // every thread sums in part order: same value everywhere, no atomics
    for (int c = 0; c < np; ++c) l_star = fmaf(l_s[c], w_s[c], l_star);
    const float inv = l_star > 0.f ? out_scale / l_star : 0.f;
    for (int d = tid; d < D; d += kCombineThreads) {
        float acc = 0.f;
        const float* src = o_part + row0 * D + d;
        int c_first = 0;
        if (d == d0) {
#pragma unroll
            for (int c = 0; c < kEarly; ++c)
                if (c < np) acc = fmaf(early[c], w_s[c], acc);
            c_first = kEarly;
        }
#pragma unroll 4
        for (int c = c_first; c < np; ++c) acc = fmaf(src[c * part_rows * D], w_s[c], acc);
        store_elem(out + static_cast<size_t>(tok) * out_stride + static_cast<size_t>(head) * D + d, acc * inv);
    }
}

// Merge of a split prefill (bf16 output, D = 128, every row has the same few parts): many rows, few parts, so a row
// takes 32 threads (four head-dim elements each, 16-byte loads of a part's row, one 8-byte store) and a workgroup eight
// rows; the parts are added in part order with the arithmetic of combine_kernel, so both give the same bits.
constexpr int kSplitRowsPerWg = 8;
__global__ __launch_bounds__(32 * kSplitRowsPerWg) void combine_splits_kernel(const float* __restrict__ o_part,
                                                                              const float* __restrict__ ml_part,
                                                                              int64_t rows, int hq_l, int n_parts,
                                                                              uint16_t* __restrict__ out, int64_t out_stride,
                                                                              float out_scale) {
    constexpr int D = 128;
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const int64_t row = static_cast<int64_t>(blockIdx.x) * kSplitRowsPerWg + (threadIdx.x >> 5);
    if (row >= rows) return;
    const int q4 = threadIdx.x & 31;
    const float* o_row = o_part + row * D + 4 * q4;
    const size_t part_stride = static_cast<size_t>(rows) * D;
    // the first parts' rows are requested before the weights are known
    constexpr int kEarly = 4;
    f32x4 early[kEarly];
#pragma unroll
    for (int c = 0; c < kEarly; ++c) early[c] = c < n_parts ? *reinterpret_cast<const f32x4*>(o_row + c * part_stride) : f32x4{0.f, 0.f, 0.f, 0.f};
    float m_star = -INFINITY;
    for (int c = 0; c < n_parts; ++c) m_star = fmaxf(m_star, ml_part[(c * rows + row) * 2]);
    float l_star = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    auto add_part = [&](int c, f32x4 v) {
        const f32x2 ml = *reinterpret_cast<const f32x2*>(ml_part + (c * rows + row) * 2);
        const float w = (ml[0] == -INFINITY) ? 0.f : exp2f(ml[0] - m_star);
        l_star = fmaf(ml[1], w, l_star);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = fmaf(v[e], w, acc[e]);
    };
#pragma unroll
    for (int c = 0; c < kEarly; ++c)
        if (c < n_parts) add_part(c, early[c]);
#pragma unroll 4
    for (int c = kEarly; c < n_parts; ++c) add_part(c, *reinterpret_cast<const f32x4*>(o_row + c * part_stride));
    const float inv = l_star > 0.f ? out_scale / l_star : 0.f;
    const int64_t tok = row / hq_l;
    const int head = static_cast<int>(row - tok * hq_l);
    uint16_t* dst = out + tok * out_stride + static_cast<int64_t>(head) * D + 4 * q4;
    uint16_t h[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) store_elem(&h[e], acc[e] * inv);
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    *reinterpret_cast<u32x2_t*>(dst) = u32x2_t{static_cast<uint32_t>(h[0]) | (static_cast<uint32_t>(h[1]) << 16),
                                               static_cast<uint32_t>(h[2]) | (static_cast<uint32_t>(h[3]) << 16)};
}

// Merge for the flat decode kernel (bf16 output, D = 128; out_scale = v_scale of an FP8 cache, else 1): one workgroup of one or four thread groups
// per output row; group pg sums the parts c = pg, pg + groups, ... for its 128 head-dim elements (with
// four groups sixteen partial rows are in flight per element) and the sums are added in group order.
// Four groups pay off when rows are few and parts many (small batches), one when it is the reverse.  The parts of a
// row are the partial rows (plan[pair].x + c) * G + head % G, c < plan[pair].y.
template <int kFlatCombineGroups>
__global__ __launch_bounds__(128 * kFlatCombineGroups) void combine_flat_kernel(
    const float* __restrict__ o_part, const float* __restrict__ ml_part, const int2* __restrict__ plan, int hq_l, int G,
    uint16_t* __restrict__ out, int64_t out_stride, float out_scale) {
    constexpr int D = 128, kThreadsF = 128 * kFlatCombineGroups;
    __shared__ float w_s[kCombineMaxParts];
    __shared__ float l_s[kCombineMaxParts];
    __shared__ float red_s[kThreadsF / 64];
    __shared__ float acc_s[kFlatCombineGroups][D];
    __shared__ float lsum_s[kFlatCombineGroups];
    const int row = blockIdx.x;  // sequence * hq_l + head
    const int tok = row / hq_l, head = row % hq_l;
    const int2 e = plan[tok * (hq_l / G) + head / G];
    const int np = min(e.y, kCombineMaxParts);
    const size_t row0 = static_cast<size_t>(e.x) * G + head % G;
    const int tid = threadIdx.x, d = tid & (D - 1), pg = tid >> 7;
    // this thread's first four parts are requested before the weights are known
    float early[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int c = pg + kFlatCombineGroups * x;
        early[x] = c < np ? o_part[(row0 + static_cast<size_t>(c) * G) * D + d] : 0.f;
    }
    float m_loc = -INFINITY;
    for (int c = tid; c < np; c += kThreadsF) {
        const float m_c = ml_part[(row0 + static_cast<size_t>(c) * G) * 2];
        w_s[c] = m_c;
        l_s[c] = ml_part[(row0 + static_cast<size_t>(c) * G) * 2 + 1];
        m_loc = fmaxf(m_loc, m_c);
    }
    m_loc = wave_max(m_loc);
    if ((tid & 63) == 0) red_s[tid >> 6] = m_loc;
    __syncthreads();
    float m_star = red_s[0];
#pragma unroll
    for (int w = 1; w < kThreadsF / 64; ++w) m_star = fmaxf(m_star, red_s[w]);
    for (int c = tid; c < np; c += kThreadsF) {
        const float m_c = w_s[c];
        w_s[c] = (m_c == -INFINITY) ? 0.f : exp2f(m_c - m_star);
    }
    __syncthreads();
    float acc = 0.f, lsum = 0.f;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int c = pg + kFlatCombineGroups * x;
        if (c < np) {
            acc = fmaf(early[x], w_s[c], acc);
            lsum = fmaf(l_s[c], w_s[c], lsum);
        }
    }
#pragma unroll 4
    for (int c = pg + 4 * kFlatCombineGroups; c < np; c += kFlatCombineGroups) {
        acc = fmaf(o_part[(row0 + static_cast<size_t>(c) * G) * D + d], w_s[c], acc);
        lsum = fmaf(l_s[c], w_s[c], lsum);
    }
    acc_s[pg][d] = acc;
    if (d == 0) lsum_s[pg] = lsum;
    __syncthreads();
    if (pg == 0) {
        float a = acc_s[0][d], l = lsum_s[0];
#pragma unroll
        for (int g2 = 1; g2 < kFlatCombineGroups; ++g2) {
            a += acc_s[g2][d];
            l += lsum_s[g2];
        }
        const float inv = l > 0.f ? out_scale / l : 0.f;
        store_elem(out + static_cast<size_t>(tok) * out_stride + static_cast<size_t>(head) * D + d, a * inv);
    }
}

}  // namespace

hipError_t launch_combine_flat(const float* o_part, const float* ml_part, const int2* plan, int num_seqs, int hq_l, int G,
                               void* out, int64_t out_stride, float out_scale, hipStream_t st) {
    const int64_t rows = static_cast<int64_t>(num_seqs) * hq_l;
    if (rows == 0) return hipSuccess;
    if (rows >= 1024)
        combine_flat_kernel<1><<<static_cast<unsigned>(rows), 128, 0, st>>>(o_part, ml_part, plan, hq_l, G,
                                                                            static_cast<uint16_t*>(out), out_stride, out_scale);
    else
        combine_flat_kernel<4><<<static_cast<unsigned>(rows), 512, 0, st>>>(o_part, ml_part, plan, hq_l, G,
                                                                            static_cast<uint16_t*>(out), out_stride, out_scale);
    return hipGetLastError();
}

hipError_t launch_attn_generic(const void* q, const void* cache, const int32_t* block_table,
                               const int32_t* cu_seqlens_q, const int32_t* seq_lens, int num_seqs, int total_q,
                               void* out, const AttnShape& a, hipStream_t st) {
    const int64_t rows = static_cast<int64_t>(total_q) * a.hq_l;
    if (rows == 0) return hipSuccess;
    const unsigned grid = static_cast<unsigned>((rows + kWaves - 1) / kWaves);
    if (a.kv_fp8()) {
        if (a.elem == 2)
            attn_rows_kernel<uint16_t, uint8_t><<<grid, kWaves * 64, 0, st>>>(
                static_cast<const uint16_t*>(q), static_cast<const uint8_t*>(cache), block_table, cu_seqlens_q, seq_lens,
                num_seqs, total_q, static_cast<uint16_t*>(out), a);
        else
            attn_rows_kernel<float, uint8_t><<<grid, kWaves * 64, 0, st>>>(
                static_cast<const float*>(q), static_cast<const uint8_t*>(cache), block_table, cu_seqlens_q, seq_lens,
                num_seqs, total_q, static_cast<float*>(out), a);
    } else if (a.elem == 2) {
        attn_rows_kernel<uint16_t, uint16_t><<<grid, kWaves * 64, 0, st>>>(
            static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(cache), block_table, cu_seqlens_q, seq_lens,
            num_seqs, total_q, static_cast<uint16_t*>(out), a);
    } else {
        attn_rows_kernel<float, float><<<grid, kWaves * 64, 0, st>>>(static_cast<const float*>(q),
                                                                   static_cast<const float*>(cache), block_table,
                                                                   cu_seqlens_q, seq_lens, num_seqs, total_q,
                                                                   static_cast<float*>(out), a);
    }
    return hipGetLastError();
}

hipError_t launch_combine(const float* o_part, const float* ml_part, int n_rows, int hq_l, int D, int n_parts,
                          int mode, const int32_t* seq_lens, int chunk, void* out, int64_t out_stride, int elem,
                          float out_scale, hipStream_t st) {
    const int64_t rows = static_cast<int64_t>(n_rows) * hq_l;
    if (rows == 0) return hipSuccess;
    if (elem == 2 && D == 128 && mode == 0 && n_parts <= kCombineMaxParts && (out_stride % 4) == 0) {
        combine_splits_kernel<<<static_cast<unsigned>((rows + kSplitRowsPerWg - 1) / kSplitRowsPerWg), 32 * kSplitRowsPerWg, 0, st>>>(
            o_part, ml_part, rows, hq_l, n_parts, static_cast<uint16_t*>(out), out_stride, out_scale);
        return hipGetLastError();
    }
    if (elem == 2)
        combine_kernel<uint16_t><<<static_cast<unsigned>(rows), 128, 0, st>>>(
            o_part, ml_part, n_rows, hq_l, D, n_parts, mode, seq_lens, chunk, static_cast<uint16_t*>(out), out_stride,
            out_scale);
    else
        combine_kernel<float><<<static_cast<unsigned>(rows), 128, 0, st>>>(o_part, ml_part, n_rows, hq_l, D, n_parts,
                                                                          mode, seq_lens, chunk,
                                                                          static_cast<float*>(out), out_stride, out_scale);
    return hipGetLastError();
}

}  // namespace shiftattn
