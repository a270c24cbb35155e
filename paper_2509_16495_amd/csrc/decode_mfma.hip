// Paged decode attention, split over the context (Algorithm 1 boxed line for decode rows; the
// paper's observation that decoding re-reads the whole KV cache per token and ends up bound by
// memory bandwidth, Sec. 4.3).  bf16 cache, head_dim 128, up to 16 query heads per KV head.
//
// Work decomposition: one workgroup per (sequence, KV head, 512-token chunk of the context); its
// four wavefronts take 32-token groups (two cache blocks) round-robin.  All query heads of the
// GQA group ride in the 16-wide N dimension of a 16x16x32 bf16 MFMA, so every K and V byte is
// read from HBM once per (sequence, KV head) and used for all heads.
//
// Per group a lane issues sixteen independent 16-byte loads (8 for K, 8 for V) directly in MFMA
// operand layout - no LDS staging:
//   S^T[token][head]  = K[token][:] . Q^T[:][head]        A = K rows,   B = Q^T (registers)
//   O^T[d][head]     += V^T[d][token] . P^T[token][head]   A = V^T rows, B = P^T (from S^T regs)
// K is stored token-major and V dimension-major in the cache, so both A operands are contiguous
// 16-byte pieces.  Tokens are assigned to MFMA rows so that the eight S^T values a lane holds
// (two 16-token tiles x four rows) are eight consecutive tokens: exactly the k-slice of P^T the
// second MFMA needs from that lane, and exactly one 16-byte piece of a V^T row.
//
// Each workgroup writes one un-normalised partial (max, sum, O) per head; launch_combine merges
// the chunks of a sequence in chunk order, so results do not depend on scheduling.
#include "internal.h"

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

__global__ __launch_bounds__(kWaves * 64, 2) void decode_splitk_kernel(
    const uint16_t* __restrict__ q, int64_t q_stride, const uint16_t* __restrict__ cache,
    const int32_t* __restrict__ block_table, int max_blocks, const int32_t* __restrict__ seq_lens,
    float* __restrict__ o_part, float* __restrict__ ml_part, int num_seqs, int hq_l, int hkv_l, float c) {
    const int chunk = blockIdx.x, s = blockIdx.y, g = blockIdx.z;
    const int ctx = seq_lens[s];
    const int t_begin = chunk * kDecodeChunk;
    if (t_begin >= ctx) return;  // uniform for the workgroup
    const int t_end = min(ctx, t_begin + kDecodeChunk);
    const int n_groups = (t_end - t_begin + kGroup - 1) / kGroup;
    const int G = hq_l / hkv_l;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int col = lane & 15;   // MFMA column: query head of the group / row index of A operands
    const int grp = lane >> 4;   // k-slice of the MFMA operands held by this lane

    __shared__ float o_s[kWaves][16][kOPad];
    __shared__ float m_s[kWaves][16];
    __shared__ float l_s[kWaves][16];

    // Q^T as B operand: column = head, k-slice = head-dim elements 8*(grp + 4*kk) .. +8
    bf16x8 qf[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (col < G)
            v = *reinterpret_cast<const u32x4*>(q + static_cast<size_t>(s) * q_stride +
                                                static_cast<size_t>(g * G + col) * kD + 8 * (grp + 4 * kk));
        qf[kk] = as_bf16x8(v);
    }

    const int32_t* table = block_table + static_cast<size_t>(s) * max_blocks;
    const int last_block = (ctx - 1) / kBlockSize;
    // token (within the 32-token group) whose K row this lane feeds into S^T tile a; tile b is +4
    const int tau_a = ((col >> 2) << 3) + (col & 3);
    const int k_sel = tau_a >> 4;                       // which of the group's two blocks
    const int k_off_a = tau_a & 15;
    const int v_sel = grp >> 1;                         // block holding tokens 8*grp .. 8*grp+7
    const int v_off = 8 * (grp & 1);

    auto load_group = [&](int gi, GroupFrags& f) {
        const int b0 = (t_begin + gi * kGroup) / kBlockSize;
        const int64_t blk0 = table[b0];
        const int64_t blk1 = table[min(b0 + 1, last_block)];
        const uint16_t* kbase = cache + cache_part_offset(k_sel ? blk1 : blk0, g, 0, hkv_l, kD);
        const uint16_t* vbase = cache + cache_part_offset(v_sel ? blk1 : blk0, g, 1, hkv_l, kD);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            f.k[kk] = *reinterpret_cast<const u32x4*>(kbase + k_off_a * kD + 8 * (grp + 4 * kk));
            f.k[4 + kk] = *reinterpret_cast<const u32x4*>(kbase + (k_off_a + 4) * kD + 8 * (grp + 4 * kk));
        }
#pragma unroll
        for (int mt = 0; mt < 8; ++mt)
            f.v[mt] = *reinterpret_cast<const u32x4*>(vbase + (16 * mt + col) * kBlockSize + v_off);
    };

    f32x4 o[8];
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) o[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY;  // running max of raw logits of this lane's head
    float l_run = 0.f;        // this lane's share of the running sum

    GroupFrags cur, nxt;
    if (wave < n_groups) load_group(wave, cur);
    for (int gi = wave; gi < n_groups; gi += kWaves) {
        const bool has_next = gi + kWaves < n_groups;
        if (has_next) load_group(gi + kWaves, nxt);

        f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur.k[kk]), qf[kk], sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur.k[4 + kk]), qf[kk], sb, 0, 0, 0);
        }
        // this lane now holds logits of tokens t0 + 8*grp + {0..3} (sa) and + {4..7} (sb)
        const int t0 = t_begin + gi * kGroup + 8 * grp;
        const int n_valid = t_end - t0;  // tokens of this lane's slice inside the context (may be <= 0 or >= 8)
        if (t_begin + (gi + 1) * kGroup > t_end) {  // last, partial group of the context: uniform branch
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (r >= n_valid) sa[r] = -INFINITY;
                if (4 + r >= n_valid) sb[r] = -INFINITY;
            }
            // cache slots past the context hold arbitrary bits: clear them so that 0 * x stays 0
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t mask = n_valid > 2 * w + 1 ? 0xFFFFFFFFu : (n_valid > 2 * w ? 0x0000FFFFu : 0u);
#pragma unroll
                for (int mt = 0; mt < 8; ++mt) cur.v[mt][w] &= mask;
            }
        }
        float mx = fmaxf(fmaxf(fmaxf(sa[0], sa[1]), fmaxf(sa[2], sa[3])), fmaxf(fmaxf(sb[0], sb[1]), fmaxf(sb[2], sb[3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);  // finite: every group holds at least one context token
        const float alpha = exp2f((m_run - m_new) * c);
        const float mc = m_new * c;
        float pa[4], pb[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            pa[r] = exp2f(fmaf(sa[r], c, -mc));
            pb[r] = exp2f(fmaf(sb[r], c, -mc));
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
            o[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur.v[mt]), pf, o[mt], 0, 0, 0);
        }
        if (has_next) cur = nxt;
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);

    // merge the four wavefronts through LDS; O^T row d = 16*mt + 4*grp + r, column = head
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) o_s[wave][col][16 * mt + 4 * grp + r] = o[mt][r];
    if (grp == 0) {
        m_s[wave][col] = m_run * c;  // -inf when this wavefront had no group
        l_s[wave][col] = l_run;
    }
    __syncthreads();
    const size_t part_row0 = (static_cast<size_t>(chunk) * num_seqs + s) * hq_l + static_cast<size_t>(g) * G;
    for (int idx = threadIdx.x; idx < G * kD; idx += kWaves * 64) {
        const int head = idx / kD, d = idx % kD;
        float m_star = m_s[0][head];  // wavefront 0 always has a group
#pragma unroll
        for (int w = 1; w < kWaves; ++w) m_star = fmaxf(m_star, m_s[w][head]);
        float acc = 0.f, l_star = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float wgt = exp2f(m_s[w][head] - m_star);  // exp2(-inf) = 0 for idle wavefronts
            acc += o_s[w][head][d] * wgt;
            l_star += l_s[w][head] * wgt;
        }
        o_part[(part_row0 + head) * kD + d] = acc;
        if (d == 0) {
            ml_part[(part_row0 + head) * 2] = m_star;
            ml_part[(part_row0 + head) * 2 + 1] = l_star;
        }
    }
}

inline int max_chunks_of(int max_seq_len) { return (max_seq_len + kDecodeChunk - 1) / kDecodeChunk; }

}  // namespace

bool decode_mfma_supported(const AttnShape& a) {
    return a.elem == 2 && a.D == kD && a.hq_l % a.hkv_l == 0 && a.hq_l / a.hkv_l <= 16;
}

size_t decode_mfma_workspace(int num_seqs, int max_seq_len, const AttnShape& a) {
    const size_t rows = static_cast<size_t>(max_chunks_of(max_seq_len)) * num_seqs * a.hq_l;
    return rows * (kD + 2) * sizeof(float);
}

hipError_t launch_decode_mfma(const void* q, const void* cache, const int32_t* block_table, const int32_t* seq_lens,
                              int num_seqs, int max_seq_len, void* out, void* workspace, const AttnShape& a,
                              hipStream_t st) {
    if (num_seqs == 0 || max_seq_len <= 0) return hipSuccess;
    const int max_chunks = max_chunks_of(max_seq_len);
    const size_t rows = static_cast<size_t>(max_chunks) * num_seqs * a.hq_l;
    float* o_part = static_cast<float*>(workspace);
    float* ml_part = o_part + rows * kD;
    const float c = a.scale * 1.4426950408889634f;
    dim3 grid(max_chunks, num_seqs, a.hkv_l);
    decode_splitk_kernel<<<grid, kWaves * 64, 0, st>>>(static_cast<const uint16_t*>(q), a.q_stride,
                                                      static_cast<const uint16_t*>(cache), block_table, a.max_blocks,
                                                      seq_lens, o_part, ml_part, num_seqs, a.hq_l, a.hkv_l, c);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_combine(o_part, ml_part, num_seqs, a.hq_l, kD, max_chunks, 1, seq_lens, kDecodeChunk, out,
                          a.out_stride, a.elem, st);
}

}  // namespace shiftattn
