// Internal launch interface between the C-ABI front end (api.hip) and the kernel files.
// Every launcher only enqueues on the given stream and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace shiftattn {

constexpr int kBlockSize = 16;         // tokens per KV-cache block
constexpr int kPrefillKvTile = 64;     // keys per prefill inner-loop step
constexpr int kMaxParts = 1024;        // most partial results the merge kernel takes per output row

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte vector

struct XchgShape {
    int P, h, h_kv, hq_l, hkv_l;  // heads in elements of one head vector
    int vec_per_head;             // 16-byte vectors per head vector (D * elem_size / 16)
    int T, T_pad;
};

struct AttnShape {
    int hq_l, hkv_l, D, elem;     // elem: bytes per element (2 = bf16, 4 = f32)
    int num_blocks, max_blocks;
    float scale;
    int64_t q_stride, kv_stride, out_stride;  // in elements
    int kv_elem;                  // bytes per cache element: elem, or 1 for an FP8 E4M3 cache
    float k_scale, v_scale;       // FP8 cache: value = code value * scale (1 otherwise)
    bool kv_fp8() const { return kv_elem == 1; }
};

// layout_kernels.hip
hipError_t launch_pack(const void* qkv, void* send, const XchgShape& s, hipStream_t st);
hipError_t launch_unpack(const void* recv, void* out, const XchgShape& s, hipStream_t st);
hipError_t launch_kv_write(const void* k_new, const void* v_new, const int64_t* slots, int n_tokens,
                           void* cache, const AttnShape& a, hipStream_t st);
// D = 128: the FP8 E4M3 cache blocks block_table[s][i], i < ceil(seq_lens[s] / 16), widened to bf16 at
// scratch block s * nb + i (same K | V^T arrangement); table_out[s][i] = s * nb + i for all i < nb.
hipError_t launch_fp8_blocks_to_bf16(const void* cache_fp8, const int32_t* block_table, int max_blocks,
                                     const int32_t* seq_lens, int num_seqs, int nb, int hkv_l, void* scratch_bf16,
                                     int32_t* table_out, hipStream_t st);

// attn_generic.hip : any dtype / head_dim / head ratio, one wavefront per (token, head) row
hipError_t launch_attn_generic(const void* q, const void* cache, const int32_t* block_table,
                               const int32_t* cu_seqlens_q /*null: one token per sequence*/,
                               const int32_t* seq_lens, int num_seqs, int total_q, void* out,
                               const AttnShape& a, hipStream_t st);

// Merge of split-context partial results (shared by decode and split prefill).
// Partials: o[part][row][D] fp32 un-normalised, ml[part][row][2] = (max logit * log2e*scale, sum).
// mode 0: every row has n_parts parts.  mode 1 (decode): row = (sequence, head), the number of
// parts of a row is ceil(seq_lens[sequence] / chunk).
hipError_t launch_combine(const float* o_part, const float* ml_part, int n_rows, int hq_l, int D,
                          int n_parts, int mode, const int32_t* seq_lens, int chunk, void* out,
                          int64_t out_stride, int elem, float out_scale, hipStream_t st);

// Merge for the flat decode kernel (bf16, D = 128): see combine_flat_kernel.
hipError_t launch_combine_flat(const float* o_part, const float* ml_part, const int2* plan, int num_seqs, int hq_l, int G,
                               void* out, int64_t out_stride, float out_scale, hipStream_t st);

// decode_mfma.hip : bf16 q/out, D = 128, hq_l/hkv_l <= 16; cache bf16 or FP8 E4M3
bool decode_mfma_supported(const AttnShape& a, int num_seqs, int max_seq_len);
size_t decode_mfma_workspace(int num_seqs, int max_seq_len, const AttnShape& a);
// k_new / v_new / slots non-null: the kernel also appends the new token of every sequence (only where
// decode_mfma_appends() says so; the caller then launches no separate K/V write)
bool decode_mfma_appends(int num_seqs, const AttnShape& a);
hipError_t launch_decode_mfma(const void* q, const void* k_new, const void* v_new, const int64_t* slots, void* cache,
                              const int32_t* block_table, const int32_t* seq_lens, int num_seqs, int max_seq_len,
                              void* out, void* workspace, const AttnShape& a, hipStream_t st);

// prefill_mfma.hip : bf16 q/out, D = 128; cache bf16, or FP8 E4M3 widened into workspace first
bool prefill_mfma_supported(const AttnShape& a, int num_seqs, int max_seq_len);
size_t prefill_mfma_workspace(int num_seqs, int total_q, int max_q_len, int max_seq_len, const AttnShape& a);
hipError_t launch_prefill_mfma(const void* q, const void* cache, const int32_t* block_table,
                               const int32_t* cu_seqlens_q, const int32_t* seq_lens, int num_seqs,
                               int total_q, int max_q_len, int max_seq_len, void* out, void* workspace,
                               const AttnShape& a, hipStream_t st);

// prefill_mfma64.hip : the same operation on 256-column workgroup tiles, one 64-column wavefront per SIMD; bf16 cache
struct Prefill64Plan {
    int tile_tokens, pair_ranks, n_splits;  // pair_ranks: workgroups per (sequence, KV head, key range)
    bool paired;                            // a workgroup takes two tiles of a sequence (heaviest with lightest)
    bool rotate;                            // rotate_sequences_over_dies() of the batch
    long workgroups;
    double model_seconds;  // launch_model_seconds of this plan
    double model_with_passes;  // the same plus what the passes of a compute unit cost around their key loops
};
// Rough duration of a prefill launch, used only to choose between plans: `wgs` workgroups (one per compute unit at a
// time) of `cols` columns each walk `walks` x max_seq_len keys cut into `splits` ranges; ranges beyond one cost a merge
// pass.
inline double launch_model_seconds(long wgs, int splits, int cols, int total_q, int max_seq_len, int hq_l, double walks) {
    const double unit = walks * 4.0 * 128 * cols * static_cast<double>(max_seq_len) / 3.9e12;  // one workgroup at 1 PFLOP/s per chip
    const double merge = 2.0 * total_q * hq_l * 130 * 4 / 4.0e12;                     // partials written and read back, per range
    const double load = static_cast<double>(wgs) * splits / 256.0;
    // equal workgroups are dispatched as compute units fall free: whole rounds while they are few, half a round of tail
    // once their durations have drifted apart
    const double whole = static_cast<double>(static_cast<long>(load + 0.999999));
    const double rounds = load <= 1.0 ? 1.0 : (whole < load + 0.5 ? whole : load + 0.5);
    return rounds / splits * unit + (splits > 1 ? splits * merge + 5.0e-6 : 0.0);
}
// Keys a workgroup walks when it takes a sequence's tiles in pairs (heaviest with lightest), in units of the context: one
// walk for a prefill from nothing (tile i sees i + 1 tiles' worth of keys, its partner the rest), two for a short chunk
// behind a long context (both tiles see nearly all of it).
inline double paired_walks(int max_q_len, int max_seq_len) {
    return max_seq_len > 0 ? 2.0 - static_cast<double>(max_q_len < max_seq_len ? max_q_len : max_seq_len) / max_seq_len : 1.0;
}
// The batch counted in sequences of its longest chunk (the lengths themselves are on the device; the host knows their
// sum and their maximum): what the workgroups of a launch planned for the longest amount to when many are light or empty.
inline double longest_chunk_equivalents(int num_seqs, int total_q, int max_q_len) {
    return max_q_len > 0 && total_q < static_cast<double>(num_seqs) * max_q_len ? static_cast<double>(total_q) / max_q_len
                                                                                : static_cast<double>(num_seqs);
}
// Workgroup i of a launch runs on die i % 8.  The prefill kernels number their workgroups (tile rank, key range) x
// (sequence, head), so when the (sequence, head) count is a multiple of eight every workgroup of a sequence lands on the
// same die: good while the sequences are alike (a die's L2 holds the K/V of its sequences only), and a 32-CU bottleneck
// for a long prompt among short ones (measured: one 4096-token prompt with seven of 700 tokens took twice the time of
// the long prompt alone).  Batches whose chunks are far from equal, and whose (sequence, head) count is a multiple of
// four (a sequence then sees one or two dies), therefore rotate the (sequence, head) index by the (tile rank, key range)
// index; other counts spread by themselves, and rotating them only costs L2 hits.
inline bool rotate_sequences_over_dies(int num_seqs, int heads, int total_q, int max_q_len) {
    return num_seqs > 1 && (static_cast<long>(num_seqs) * heads) % 4 == 0 &&
           longest_chunk_equivalents(num_seqs, total_q, max_q_len) < 0.75 * num_seqs;
}
bool prefill_mfma64_supported(const AttnShape& a);
Prefill64Plan prefill_mfma64_plan(int num_seqs, int total_q, int max_q_len, int max_seq_len, const AttnShape& a,
                                  int forced_splits);
size_t prefill_mfma64_workspace(int total_q, const Prefill64Plan& pl, const AttnShape& a);
// c: softmax scale in exp2 units (times k_scale), out_scale: factor on the normalised output (v_scale, else 1)
hipError_t launch_prefill_mfma64(const void* q, const void* cache, const int32_t* block_table, int max_blocks,
                                 const int32_t* cu_seqlens_q, const int32_t* seq_lens, int num_seqs, int total_q,
                                 const Prefill64Plan& pl, void* out, void* workspace, const AttnShape& a, float c,
                                 float out_scale, hipStream_t st);

// Per-device set-up of the kernels that need more dynamic LDS than the default limit (each sets the attribute of its
// kernels on the current device).  api.hip calls them once per device, under a lock, before the first launch there.
hipError_t prefill_mfma_init();
hipError_t prefill_mfma64_init();
hipError_t proj_gemm_init();
hipError_t proj_stream_init();

// Process-wide tuning switches (api.hip: shiftattn_set_option); 0 = decided per call
int option_prefill_tile();    // 0, 128 or 256
int option_prefill_splits();  // 0 or the number of key ranges
int option_prefill_pairing(); // 0, 1 (tiles in pairs) or 2 (one tile per workgroup)
int option_prefill_scaled_q();     // 1: the 256-column kernel's first attempt works on Q times the scale, re-rounded

// proj_gemm.hip : the projections in front of the first exchange and behind the second (bf16, head_dim 128)
bool qkv_proj_pack_supported(const XchgShape& s, int d_model, int elem);
bool unpack_o_proj_supported(const XchgShape& s, int d_model, int elem);
// scales non-null: the operands are FP8 E4M3 codes with one scale per token row and one per output feature
// (the result stays bf16); the XchgShape then describes the bf16 side (send buffers) or, for the receive buffers,
// their head geometry
hipError_t launch_qkv_proj_pack(const void* x, const void* w_qkv, void* send, int d_model, const XchgShape& s,
                                const float* x_scales, const float* w_scales, void* workspace, size_t workspace_bytes,
                                hipStream_t st);
hipError_t launch_unpack_o_proj(const void* recv, const void* w_o, void* out, int d_model, const XchgShape& s,
                                const float* a_scales, const float* w_scales, void* workspace, size_t workspace_bytes,
                                hipStream_t st);
// bytes of workspace that let the large-batch kernel split k over workgroups for its last (or only) round of tiles; 0: no split
size_t proj_gemm_workspace(int M_out, int N, int K, bool fp8);
// proj_stream.hip : the same two products for up to 64 token rows, organised around one pass over the weights
size_t proj_stream_workspace(int M_out, int N, int K, bool fp8);
bool proj_stream_takes(int M_out, int N, int K, bool fp8, size_t workspace_bytes);
hipError_t launch_qkv_proj_stream(const void* x, const void* w_qkv, void* send, int d_model, const XchgShape& s,
                                  const float* x_scales, const float* w_scales, void* workspace, hipStream_t st);
hipError_t launch_o_proj_stream(const void* recv, const void* w_o, void* out, int d_model, const XchgShape& s,
                                const float* a_scales, const float* w_scales, void* workspace, hipStream_t st);
// (row_base: the partial results start at this token row of the result; rows below it are not touched)
hipError_t launch_proj_finish(const float* partial, int kg, int t_rows, void* c, int M, int M_out, int N, int mode,
                              const XchgShape& s, const float* x_scales, const float* w_scales, hipStream_t st,
                              int row_base = 0);
// layout_kernels.hip : rows of bf16 values -> FP8 E4M3 codes + one float32 scale per row (amax / 448).  Element k of
// row t lies at (k / seg_len) * seg_stride + t * row_stride + k % seg_len, in `x` and in `codes` alike.
hipError_t launch_quantize_rows_fp8(const void* x, void* codes, float* scales, int rows, int cols, int seg_len,
                                    int64_t seg_stride, int64_t row_stride, hipStream_t st);

// ceilings.hip : attainable-rate probes for benchmark reports
hipError_t launch_mfma_ceiling(const void* operands, void* sink, int iters, int64_t* flops, hipStream_t st);
hipError_t launch_mfma_ceiling_fresh(const void* operands, void* sink, int iters, int64_t* flops, hipStream_t st);
hipError_t launch_hbm_read_ceiling(const void* src, size_t bytes, void* sink, int64_t* bytes_read, hipStream_t st);
hipError_t launch_hbm_copy_ceiling(const void* src, void* dst, size_t bytes, int64_t* bytes_copied, hipStream_t st);

// FP8 E4M3 codes of a / scale and b / scale in bits 0..7 and 8..15: float32 quotient, nearest code with
// ties to the even code, clamped to +-448 first so that nothing overflows, NaN quotient -> NaN code
__device__ inline uint32_t e4m3_pair(float a, float b, float scale) {
    const float qa = a / scale, qb = b / scale;
    const float ca = fminf(fmaxf(qa, -448.f), 448.f), cb = fminf(fmaxf(qb, -448.f), 448.f);
    uint32_t w = static_cast<uint32_t>(__builtin_amdgcn_cvt_pk_fp8_f32(ca, cb, 0, false)) & 0xFFFFu;
    if (qa != qa) w |= 0x7Fu;
    if (qb != qb) w |= 0x7F00u;
    return w;
}

// element offsets inside the cache: kv_cache[block][kv head][2][16*D]
__host__ __device__ inline size_t cache_part_offset(int64_t block, int g, int part, int hkv_l, int D) {
    return ((static_cast<size_t>(block) * hkv_l + g) * 2 + part) * static_cast<size_t>(kBlockSize) * D;
}

}  // namespace shiftattn
