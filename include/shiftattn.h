/*
 * shiftattn.h - C ABI of one GPU's share of an attention layer under Shift Parallelism
 * (arXiv 2509.16495), for AMD MI355X (gfx950).
 *
 * The library covers what a rank does between the QKV projection and the O projection
 * (Algorithm 1, the two SP all-to-all lines and the boxed attention line):
 *
 *   shiftattn_pack_seq2head     send side of the sequence->head all-to-all (SP mode only)
 *   shiftattn_kv_write          append new K/V rows to the paged KV cache
 *   shiftattn_prefill           causal attention of new-token chunks over the cache (fused KV append)
 *   shiftattn_decode            one-token-per-sequence attention, split over the context (fused KV append)
 *   shiftattn_mixed             a unified batch of chunks and decode rows in one call
 *   shiftattn_unpack_head2seq   receive side of the head->sequence all-to-all (SP mode only)
 *
 * and, next to the exchange, the two projections fused with its layouts (bf16, or FP8 E4M3 operands):
 *
 *   shiftattn_qkv_proj_pack[_fp8]   qkv = x * W_qkv^T written straight into the send buffers
 *   shiftattn_unpack_o_proj[_fp8]   embed = unpack(recv) * W_o^T read in place from the receive buffers
 *   shiftattn_quantize_rows_fp8 / shiftattn_quantize_recv_fp8   per-row FP8 quantisation for the above
 *
 * In TP mode (the shift configuration, SP=1) a rank calls only kv_write/prefill/decode on the
 * fused rows its own QKV projection produced; in SP mode it packs, exchanges, attends,
 * exchanges, unpacks.  Both modes drive the same attention kernels over the same cache: that
 * is the KV-cache invariance of Sec. 3.1 / 3.3.1.  The exchange itself (the wire transfer) is
 * not part of this library.
 *
 * Conventions for every entry point
 *   - Pointers named in "device" positions are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or synchronises: each call validates its arguments on the host,
 *     then only enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream).  No host-side read of device memory, so calls can be captured into a HIP graph.
 *   - Return value: SHIFTATTN_OK or a negative error code.  Arguments are validated before any
 *     launch; on error nothing has been enqueued.  shiftattn_last_error() returns a
 *     thread-local description of the last failure.  No C++ exception crosses this boundary.
 *   - Element types: SHIFTATTN_BF16 (bfloat16, 2 bytes) or SHIFTATTN_F32 (4 bytes); all
 *     tensors of one call share the type.  head_dim * element size must be a multiple of 16 and
 *     all tensor base pointers and row strides must be 16-byte aligned.
 *   - Contents of device-side index arrays (slots, block ids, lengths) are trusted: an
 *     out-of-range block id or slot is undefined behaviour.
 *
 * Paged KV cache (layout is a convention of this library; the paper only requires that it is
 * the same in SP and TP mode):
 *     kv_cache[num_blocks][num_kv_heads][2][block_size * head_dim]
 *   part 0 holds K token-major,      K[offset][d]
 *   part 1 holds V dimension-major,  V[d][offset]
 *   with offset = token position % block_size.  Slot id = block * block_size + offset.
 *   block_size is 16.  block_table[s][i] is the cache block of tokens [16 i, 16 i + 16) of
 *   sequence s; entries past the sequence's last block are never read.
 *
 * FP8 KV cache (kv_format = SHIFTATTN_KV_FP8_E4M3; Sec. 4.1 runs its long-trace experiment with
 * an FP8 KV cache and gives no format or scale rule - the rule here is this library's): the same
 * arrangement with one byte per element, an OCP FP8 E4M3 code (bias 7, no infinities, largest
 * finite 448).  A stored element stands for code_value * k_scale (K) or code_value * v_scale (V).
 * The writer computes x / scale in float32 and rounds to the nearest code, ties to the even code,
 * magnitudes beyond 448 saturating; NaN gives a NaN code.  q, k_new, v_new and out keep `dtype`.
 */
#ifndef SHIFTATTN_H
#define SHIFTATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SHIFTATTN_OK = 0,
    SHIFTATTN_EINVAL = -1,       /* null pointer, negative size, inconsistent arguments          */
    SHIFTATTN_EUNSUPPORTED = -2, /* well-formed but not built (head_dim, block_size, head ratio)  */
    SHIFTATTN_EWORKSPACE = -3,   /* workspace missing or smaller than *_workspace_bytes() says    */
    SHIFTATTN_EHIP = -4          /* the HIP runtime refused a launch                               */
};

enum { SHIFTATTN_BF16 = 0, SHIFTATTN_F32 = 1 };
enum { SHIFTATTN_KV_SAME = 0 /* cache elements have `dtype` */, SHIFTATTN_KV_FP8_E4M3 = 1 };

/* One sequence<->head exchange among P ranks (Algorithm 1: P is the SP degree of the base
 * configuration; h and h_kv are the heads a source rank holds, i.e. model heads / TP). */
typedef struct shiftattn_xchg {
    int32_t P;            /* members of the exchange group, >= 1                                  */
    int32_t num_q_heads;  /* h: query heads per source row; must be a multiple of P                */
    int32_t num_kv_heads; /* h_kv: K (and V) heads per source row; 0 = query-only rows.  Either a
                             multiple of P (each destination gets h_kv/P heads) or a divisor of P
                             (each head is replicated to P/h_kv consecutive destinations,
                             Sec. 3.2.1 "KV Cache Replication")                                    */
    int32_t head_dim;     /* D                                                                     */
    int32_t dtype;        /* SHIFTATTN_BF16 | SHIFTATTN_F32                                        */
} shiftattn_xchg;

/* The local head shard and its cache (Algorithm 1, boxed line: h/(SP*TP) heads over all n tokens). */
typedef struct shiftattn_attn {
    int32_t num_q_heads;        /* hq_l: local query heads                                         */
    int32_t num_kv_heads;       /* hkv_l: local KV heads; hq_l must be a multiple of it (GQA)      */
    int32_t head_dim;           /* D: 64 or 128 are tuned; any multiple of 8 up to 256 is accepted */
    int32_t dtype;              /* SHIFTATTN_BF16 | SHIFTATTN_F32                                  */
    int32_t block_size;         /* tokens per cache block; must be 16                              */
    int32_t num_blocks;         /* blocks in kv_cache                                              */
    int32_t max_blocks_per_seq; /* row length of block_table                                       */
    float softmax_scale;        /* multiplies q.k before the softmax (the paper leaves it implicit;
                                   1/sqrt(D) is customary)                                         */
    int64_t q_stride;           /* elements between consecutive tokens of q;   0 = hq_l*D (dense)  */
    int64_t kv_stride;          /* same for k_new and v_new;                   0 = hkv_l*D         */
    int64_t out_stride;         /* same for out;                               0 = hq_l*D          */
    int32_t kv_format;          /* SHIFTATTN_KV_SAME | SHIFTATTN_KV_FP8_E4M3 (needs head_dim % 16 == 0) */
    float k_scale;              /* FP8 cache only: value of a K element = code value * k_scale, > 0 */
    float v_scale;              /* FP8 cache only: same for V                                      */
    int32_t reserved;           /* must be 0                                                       */
} shiftattn_attn;
/* Strides let q, k_new and v_new be views into one fused receive buffer
 * [n_pad][hq_l + 2*hkv_l][D]: q = buf, k_new = buf + hq_l*D, v_new = buf + (hq_l+hkv_l)*D,
 * q_stride = kv_stride = (hq_l + 2*hkv_l)*D. */

/* ---- Algorithm 1, first SP all-to-all, send side ("fused" q|k|v exchange, Sec. 3.2.1) ----------
 * qkv  (device, in) : [T][h + 2*h_kv][D]   this rank's rows; per row: q heads, then k heads, then
 *                                          v heads, each D contiguous elements.
 * send (device, out): [P][T_pad][hq_l + 2*hkv_l][D], hq_l = h/P, hkv_l = max(1, h_kv/P)
 *                     (hkv_l = 0 when h_kv = 0).  Buffer p holds query heads [p*hq_l, (p+1)*hq_l)
 *                     followed by the K then V heads that GQA assigns to them, starting at KV head
 *                     floor(p*h_kv/P).  Rows T..T_pad-1 (padding of the batch to a multiple of the
 *                     SP degree, Sec. 3.2.1 "Load Imbalance") are written as zeros.
 * After the exchange, destination p's receive buffer is the concatenation over source ranks of
 * their send[p] and needs no further transform.
 * Errors: EINVAL for null pointers (unless the tensor is empty), T<0, T_pad<T, P<1, h%P != 0,
 * h_kv neither multiple nor divisor of P; EUNSUPPORTED for D*elem_size % 16 != 0 or more than
 * 2^31-1 16-byte vectors per tensor. */
int shiftattn_pack_seq2head(const void *qkv, void *send, int32_t T, int32_t T_pad, const shiftattn_xchg *x,
                            void *stream);

/* ---- Algorithm 1, second SP all-to-all, receive side -------------------------------------------
 * recv (device, in) : [P][T_pad][hq_l][D]  buffer p = the attention output rows this rank owns,
 *                                          computed by the rank holding head block p.
 * out  (device, out): [T][h][D] with out[t][p*hq_l + j] = recv[p][t][j]; padding rows dropped.
 * x->num_kv_heads is ignored.  Errors as for pack. */
int shiftattn_unpack_head2seq(const void *recv, void *out, int32_t T, int32_t T_pad, const shiftattn_xchg *x,
                              void *stream);

/* ---- Algorithm 1, the projections on either side of the exchange (bf16, head_dim 128) -----------
 * qkv_proj_pack: qkv = x * W_qkv^T (the line in front of the first all-to-all) written straight into
 *   the send buffers of shiftattn_pack_seq2head - same buffers, same bytes as projecting into
 *   [T][h + 2 h_kv][D] and packing, without that tensor ever existing.
 *   x (device, in)    : [T][d_model]
 *   w_qkv (device, in): [(h + 2 h_kv) * D][d_model], one row per output feature, features in the
 *                       order q heads, k heads, v heads
 *   send (device, out): [P][T_pad][hq_l + 2 hkv_l][D]; rows T..T_pad-1 zero
 *   Needs d_model % 64 == 0 and an even h + 2 h_kv (else EUNSUPPORTED).
 * unpack_o_proj: embed = unpack(recv) * W_o^T (the line behind the second all-to-all), the attention
 *   output read in place from the receive buffers of shiftattn_unpack_head2seq.
 *   recv (device, in) : [P][T_pad][hq_l][D]
 *   w_o (device, in)  : [d_model][h * D], one row per output feature
 *   out (device, out) : [T][d_model]
 *   Needs d_model % 256 == 0 (else EUNSUPPORTED).
 * fp32 accumulation, results rounded to bf16 (nearest even).  Other checks as for pack / unpack. */
int shiftattn_qkv_proj_pack(const void *x, const void *w_qkv, void *send, int32_t T, int32_t T_pad,
                            int32_t d_model, const shiftattn_xchg *xc, void *stream);
int shiftattn_unpack_o_proj(const void *recv, const void *w_o, void *out, int32_t T, int32_t T_pad,
                            int32_t d_model, const shiftattn_xchg *xc, void *stream);

/* ---- The same two projections with a workspace (Algorithm 2: the few-token steps below the threshold) ----
 * With up to 64 token rows (T_pad for qkv_proj_pack, T for unpack_o_proj) the product is one pass over the
 * weight matrix; from 17 rows on (at d_model = 8192) that pass is split over k between workgroups.  With a few
 * hundred rows the large-batch kernel has too few output tiles to fill the chip and splits k as well, and with
 * a few thousand (a prefill chunk) it does so for the last token rows when the tiles are no multiple of the
 * chip's compute units.  Either way the fp32 partial results need device memory:
 *   shiftattn_proj_workspace_bytes(rows, n_features, k): bytes for a product of `rows` token rows with a
 *     [n_features][k] weight matrix (qkv: n_features = (h + 2 h_kv) * D, k = d_model; o: n_features =
 *     d_model, k = h * D); 0 when none is needed.
 * workspace (device, scratch): at least that many bytes, 16-byte aligned; NULL / 0 is always accepted and
 *   means "use a kernel that needs none" (the calls above do exactly that) - between 17 rows and a few
 *   hundred that is up to several times slower.  Calls that share a workspace must not overlap.
 * Results are bitwise reproducible with and without a workspace, not bitwise equal between the two. */
size_t shiftattn_proj_workspace_bytes(int32_t rows, int32_t n_features, int32_t k);
int shiftattn_qkv_proj_pack_ws(const void *x, const void *w_qkv, void *send, int32_t T, int32_t T_pad,
                               int32_t d_model, const shiftattn_xchg *xc, void *workspace,
                               size_t workspace_bytes, void *stream);
int shiftattn_unpack_o_proj_ws(const void *recv, const void *w_o, void *out, int32_t T, int32_t T_pad,
                               int32_t d_model, const shiftattn_xchg *xc, void *workspace,
                               size_t workspace_bytes, void *stream);

/* ---- The same projections with FP8 E4M3 operands (Sec. 4.1: the served models are FP8) ------------
 * The paper gives no quantisation rule; this library's: a matrix row r is stored as OCP FP8 E4M3 codes
 * plus one float32 scale, scale[r] = max_k |x[r][k]| / 448 (1 for a row of zeros), code = the E4M3 code
 * nearest (ties to even) to the float32 quotient x / scale[r]; a row is a token for activations (dynamic
 * per-token scale) and an output feature for weights.  A product is
 *   y[t][f] = x_scale[t] * w_scale[f] * sum_k value(x_code[t][k]) * value(w_code[f][k]),
 * summed in fp32 by the FP8 matrix cores and rounded once to bf16.
 * quantize_rows_fp8: x [rows][cols] bf16 (device) -> codes [rows][cols] bytes, scales [rows] floats;
 *   cols % 8 == 0.  Use it for activations and, once, for weights.
 * quantize_recv_fp8: the same for the attention output as it lies in the receive buffers: row t is the
 *   concatenation over p of recv[p][t][0..hq_l-1][0..D-1]; codes come out in the same [P][T_pad][hq_l][D]
 *   arrangement (one byte per element; rows T..T_pad-1 are left untouched), scales [T].
 *   xc->dtype must be SHIFTATTN_BF16, head_dim % 8 == 0.
 * qkv_proj_pack_fp8 / unpack_o_proj_fp8: as the bf16 calls above with the operands replaced by codes and
 *   their scales; send / out stay bf16, xc describes them (dtype SHIFTATTN_BF16, head_dim 128).
 *   Same shape requirements as the bf16 calls.  All pointers device, 16-byte aligned (scales: 4). */
int shiftattn_quantize_rows_fp8(const void *x, void *codes, float *scales, int32_t rows, int32_t cols,
                                void *stream);
int shiftattn_quantize_recv_fp8(const void *recv, void *codes, float *scales, int32_t T, int32_t T_pad,
                                const shiftattn_xchg *xc, void *stream);
int shiftattn_qkv_proj_pack_fp8(const void *x_codes, const float *x_scales, const void *w_codes,
                                const float *w_scales, void *send, int32_t T, int32_t T_pad, int32_t d_model,
                                const shiftattn_xchg *xc, void *stream);
int shiftattn_unpack_o_proj_fp8(const void *recv_codes, const float *a_scales, const void *w_codes,
                                const float *w_scales, void *out, int32_t T, int32_t T_pad, int32_t d_model,
                                const shiftattn_xchg *xc, void *stream);
/* The FP8 projections with a workspace, as the bf16 forms above: up to 64 token rows are one pass over the weight
 * codes (k groups, and with them a workspace, from 33 rows on at d_model = 8192), a few hundred rows split k over
 * workgroups; the scales are applied once, after the fp32 sums of all of k are added.
 * shiftattn_proj_workspace_bytes_fp8: the size for FP8 operands (it differs from the bf16 size). */
size_t shiftattn_proj_workspace_bytes_fp8(int32_t rows, int32_t n_features, int32_t k);
int shiftattn_qkv_proj_pack_fp8_ws(const void *x_codes, const float *x_scales, const void *w_codes,
                                   const float *w_scales, void *send, int32_t T, int32_t T_pad, int32_t d_model,
                                   const shiftattn_xchg *xc, void *workspace, size_t workspace_bytes, void *stream);
int shiftattn_unpack_o_proj_fp8_ws(const void *recv_codes, const float *a_scales, const void *w_codes,
                                   const float *w_scales, void *out, int32_t T, int32_t T_pad, int32_t d_model,
                                   const shiftattn_xchg *xc, void *workspace, size_t workspace_bytes, void *stream);

/* ---- KV-cache append (Sec. 2.2: prefill initialises the cache, decoding appends to it) --------
 * k_new, v_new (device, in): [n_tokens][hkv_l][D] with row stride a->kv_stride.
 * slot_mapping (device, in): int64 [n_tokens]; token i goes to slot slot_mapping[i];
 *                            a negative slot (padding row) writes nothing.
 * kv_cache (device, in/out): see the layout above.  Untouched slots keep their bytes. */
int shiftattn_kv_write(const void *k_new, const void *v_new, const int64_t *slot_mapping, int32_t n_tokens,
                       void *kv_cache, const shiftattn_attn *a, void *stream);

/* ---- Algorithm 1, boxed line: attention of prefill chunks ---------------------------------------
 * Sequence s has q_len_s = cu_seqlens_q[s+1]-cu_seqlens_q[s] new tokens and seq_lens[s] tokens in
 * total (cached + new).  New token i sits at position pos = seq_lens[s] - q_len_s + i and attends
 * to positions 0..pos of its own sequence (causal, aligned to the end of the context, which is
 * what chunked prefill needs).  Query head j uses KV head j / (hq_l/hkv_l).
 *
 * q (device, in)            : [total_q][hq_l][D], row stride a->q_stride
 * k_new, v_new, slot_mapping: as in shiftattn_kv_write with n_tokens = total_q.  All three NULL =
 *                             the cache already holds the new tokens.  Otherwise they are written
 *                             first and the result equals "write, then attend".
 * block_table (device, in)  : int32 [num_seqs][max_blocks_per_seq]
 * cu_seqlens_q (device, in) : int32 [num_seqs + 1], cu_seqlens_q[0] = 0, non-decreasing
 * seq_lens (device, in)     : int32 [num_seqs], seq_lens[s] >= q_len_s
 * total_q, max_q_len, max_seq_len (host): total_q = cu_seqlens_q[num_seqs]; upper bounds on
 *                             q_len_s and seq_lens[s] (they size the launch; exceeding them
 *                             silently drops work)
 * out (device, out)         : [total_q][hq_l][D], row stride a->out_stride
 * workspace (device)        : at least shiftattn_prefill_workspace_bytes(...) bytes, 16-byte
 *                             aligned; may be NULL when that is 0.  Contents are scratch.
 * Arithmetic of the bf16 path: logits and outputs accumulate in fp32, the softmax (scale included)
 * runs in fp32, the probabilities are rounded to bf16 before the second product, the output once
 * at the end.  (SHIFTATTN_OPT_PREFILL_SCALED_Q trades one more rounding of Q for speed.)
 * num_seqs == 0 or total_q == 0 is a valid no-op. */
int shiftattn_prefill(const void *q, const void *k_new, const void *v_new, const int64_t *slot_mapping,
                      void *kv_cache, const int32_t *block_table, const int32_t *cu_seqlens_q,
                      const int32_t *seq_lens, int32_t num_seqs, int32_t total_q, int32_t max_q_len,
                      int32_t max_seq_len, void *out, void *workspace, size_t workspace_bytes,
                      const shiftattn_attn *a, void *stream);

/* ---- Algorithm 1, boxed line: attention of decode rows (one new token per sequence) -------------
 * Same definition with q_len_s = 1, pos = seq_lens[s] - 1.  The contexts of the batch are cut into
 * pieces processed in parallel (equal shares of all tokens per wavefront); partial results are
 * merged in a fixed order, so results are bitwise reproducible from run to run.
 * q, out: [num_seqs][hq_l][D]; k_new/v_new/slot_mapping: n_tokens = num_seqs (or all NULL).
 * seq_lens[s] <= 0 marks a padding row (an engine that replays captured graphs pads its batches,
 * Sec. 3.4): its output rows are zero, its table row is not read, and its slot must be negative.
 * slot_mapping[s], when not negative, must be the slot of position seq_lens[s] - 1 of sequence s as
 * block_table maps it (the append of a decode step): the tuned kernel writes the new token and attends to
 * it in one launch and does not re-read that slot through the table. */
int shiftattn_decode(const void *q, const void *k_new, const void *v_new, const int64_t *slot_mapping,
                     void *kv_cache, const int32_t *block_table, const int32_t *seq_lens, int32_t num_seqs,
                     int32_t max_seq_len, void *out, void *workspace, size_t workspace_bytes,
                     const shiftattn_attn *a, void *stream);

/* ---- shiftattn_decode for callers that cannot allocate -------------------------------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc: the same
 * operation, arguments and results as shiftattn_decode, but the split partials go into device memory the
 * library itself holds (a file-scope array of SHIFTATTN_STATIC_SCRATCH_BYTES on every GPU the library
 * runs on, until the process ends) instead of a caller-provided workspace.  The call allocates and frees
 * nothing.  A batch whose shiftattn_decode_workspace_bytes() exceeds SHIFTATTN_STATIC_SCRATCH_BYTES is
 * refused with SHIFTATTN_EWORKSPACE before anything is enqueued (256 sequences of 8 query heads per KV
 * head need 9.6 MB).  Nothing in the array has to start at zero: every partial row the merge reads was
 * written by the same call.  All calls on one GPU share the one array: two calls that overlap in time
 * on the same GPU (different streams, or different host threads without ordering) race; calls on one
 * stream are ordered and safe.  The first call on a device looks the array's address up (that device must
 * be current, as for every call). */
#define SHIFTATTN_STATIC_SCRATCH_BYTES (16u << 20)
int shiftattn_decode_static(const void *q, const void *k_new, const void *v_new, const int64_t *slot_mapping,
                            void *kv_cache, const int32_t *block_table, const int32_t *seq_lens, int32_t num_seqs,
                            int32_t max_seq_len, void *out, const shiftattn_attn *a, void *stream);

/* ---- Algorithm 1, boxed line, on a unified batch: prefill chunks and decode rows in one call ------
 * A chunked-prefill engine (Sec. 5, related work on chunked prefill) puts both kinds of rows into one
 * batch.  Sequences 0 .. num_prefill_seqs-1 carry the chunks (any q_len, described by cu_seqlens_q
 * [num_prefill_seqs + 1]); the num_decode_seqs sequences after them carry one new token each.
 * Row order of q, out, k_new, v_new, slot_mapping: the total_prefill_q rows of the chunks, then one
 * row per decode sequence.  block_table and seq_lens cover all sequences in that order.
 * The K/V of all rows is written once, then each kind of row runs through its kernel; the result is
 * the same as shiftattn_prefill on the first part followed by shiftattn_decode on the second.
 * max_prefill_seq_len / max_decode_seq_len bound seq_lens of the two parts.  The workspace is shared
 * by the two parts: at least shiftattn_mixed_workspace_bytes(...).  Either part may be empty. */
int shiftattn_mixed(const void *q, const void *k_new, const void *v_new, const int64_t *slot_mapping,
                    void *kv_cache, const int32_t *block_table, const int32_t *cu_seqlens_q,
                    const int32_t *seq_lens, int32_t num_prefill_seqs, int32_t total_prefill_q,
                    int32_t max_q_len, int32_t max_prefill_seq_len, int32_t num_decode_seqs,
                    int32_t max_decode_seq_len, void *out, void *workspace, size_t workspace_bytes,
                    const shiftattn_attn *a, void *stream);

/* Workspace sizes (host only, no GPU work).  Return 0 when no workspace is needed; SIZE_MAX on
 * invalid arguments. */
size_t shiftattn_prefill_workspace_bytes(int32_t num_seqs, int32_t total_q, int32_t max_q_len,
                                         int32_t max_seq_len, const shiftattn_attn *a);
size_t shiftattn_decode_workspace_bytes(int32_t num_seqs, int32_t max_seq_len, const shiftattn_attn *a);
size_t shiftattn_mixed_workspace_bytes(int32_t num_prefill_seqs, int32_t total_prefill_q, int32_t max_q_len,
                                       int32_t max_prefill_seq_len, int32_t num_decode_seqs,
                                       int32_t max_decode_seq_len, const shiftattn_attn *a);

/* ---- Host-side index helpers (no GPU work) -------------------------------------------------------
 * Head block held by global rank `rank` in base configuration (SP=sp, TP=tp): TP groups are runs
 * of consecutive ranks, SP groups take every tp-th rank, so the block is (rank % tp)*sp + rank/tp.
 * The shift configuration (1, sp*tp) must shard its weights in this order to keep the cache valid
 * (Sec. 3.3.1; for (3,2) the ranks in block order are 0,2,4,1,3,5).  Returns -1 on bad arguments. */
int32_t shiftattn_head_block(int32_t sp, int32_t tp, int32_t rank);
/* First KV head that head block `block` of `P` uses when the source holds h_kv KV heads:
 * floor(block*h_kv/P).  Returns -1 on bad arguments. */
int32_t shiftattn_kv_head_of_block(int32_t block, int32_t P, int32_t h_kv);
/* Batch size padded up to a multiple of the SP degree (Sec. 3.2.1).  Returns -1 on bad arguments. */
int32_t shiftattn_padded_tokens(int32_t n, int32_t sp);

/* Algorithm 2 (the shift dispatcher): 1 when a batch of n_tokens runs in the base configuration
 * (SP, TP), i.e. n_tokens > threshold, 0 when it runs in the shift configuration (1, SP x TP).
 * Returns -1 on negative arguments. */
int32_t shiftattn_use_base_config(int32_t n_tokens, int32_t threshold);

/* ---- Set-up and tuning switches (for callers and benchmarks; not part of the attention path) -----------
 * shiftattn_init: optional.  Does, for the current device, the one-time set-up that the first call of an
 *   entry point would otherwise do there (kernel attributes, the address of the library's own scratch
 *   array): call it once per device before capturing calls into a HIP graph.  Thread-safe.
 * shiftattn_set_option / shiftattn_get_option: process-wide switches, 0 = the library decides per call
 *   (the default, and the fastest).  Set them before asking for workspace sizes: the sizes follow them.
 *   SHIFTATTN_OPT_PREFILL_TILE   128 | 256: which prefill kernel takes bf16 / head_dim 128 launches
 *   SHIFTATTN_OPT_PREFILL_SPLITS 1 .. 64: key ranges per column tile of those kernels
 *   SHIFTATTN_OPT_GENERIC_ONLY   1: every attention call runs the general kernel (any type / head_dim)
 *   SHIFTATTN_OPT_PREFILL_PAIRING 1 | 2: the 256-column prefill kernel takes a sequence's column tiles two per
 *                                workgroup, heaviest with lightest (1), or one per workgroup, heaviest first (2)
 *   SHIFTATTN_OPT_PREFILL_SCALED_Q 1: the 256-column prefill kernel multiplies Q by the softmax scale when a tile
 *                                fetches it, rounds it to bf16 again and takes its softmax without a reference,
 *                                so that its loop spends no instruction on scaling and shifting logits (about
 *                                4 % faster).  A logit then moves by up to 2^-9 of its value and the largest
 *                                probability of a row is no longer exactly 1: outputs of magnitude 2 and more
 *                                can land one bf16 step from the correctly rounded value.  Tiles whose softmax
 *                                sums leave [2^-40, 2^40] are recomputed on Q as given.  Off by default
 *   set returns EINVAL for an unknown option or value; get returns -1 for an unknown option. */
enum { SHIFTATTN_OPT_PREFILL_TILE = 0, SHIFTATTN_OPT_PREFILL_SPLITS = 1, SHIFTATTN_OPT_GENERIC_ONLY = 2,
       SHIFTATTN_OPT_PREFILL_PAIRING = 3, SHIFTATTN_OPT_PREFILL_SCALED_Q = 4, SHIFTATTN_OPT_COUNT = 5 };
int shiftattn_init(void);
int shiftattn_set_option(int32_t option, int32_t value);
int32_t shiftattn_get_option(int32_t option);

/* Thread-local text of the last error returned on this thread ("" if none). */
const char *shiftattn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SHIFTATTN_H */
