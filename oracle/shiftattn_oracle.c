/*
 * CPU oracle for one GPU's share of an attention layer under Shift Parallelism.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * head-shard attention path computes.  Nothing in the product path may call it;
 * only the tests, the smoke check and the CPU-baseline leg of the benchmark do.
 * It shares no code, header, table or helper with the HIP implementation.
 *
 * What it states (citations are to the paper):
 *   - softmax attention over the local heads and the full sequence
 *     (Sec. 2.2 "Transformer Architecture"; Algorithm 1, the boxed attention
 *     line), with grouped-query sharing of KV heads (Sec. 3.2.1 "GQA Extension");
 *   - the KV cache as the only state of a request, written once per token and
 *     re-read by later tokens (Sec. 2.2), in a layout that does not depend on
 *     whether the rows arrived through the SP exchange or straight from a TP
 *     shard (Sec. 3.1 "KV cache invariance");
 *   - the send-side pack of the sequence-to-head all-to-all and the
 *     receive-side unpack of the head-to-sequence all-to-all (Algorithm 1,
 *     the two SP all-to-all lines), with the fused q|k|v row of h + 2*h_kv
 *     heads, KV replication inside the send buffers when P > h_kv, and rows
 *     padded to a multiple of the SP degree (Sec. 3.2.1);
 *   - the rank -> head-block map that keeps base and shift configurations on
 *     the same head order (Sec. 3.3.1 "General KV Cache Invariance").
 *
 * All floating point work is in double over the stored input values, which are
 * widened exactly (bfloat16 and float32 both embed in double).
 *
 * Cache layout (a convention of this build; the paper fixes only that it is
 * mode-invariant):  kv_cache[num_blocks][hkv_l][2][block_size*D] where part 0
 * is K stored token-major  K[off][d]  and part 1 is V stored dimension-major
 * V[d][off]  (off = token offset in the block).
 *
 * FP8 KV cache (Sec. 4.1 names an FP8 KV cache for the long-trace experiment and
 * gives no format or scale rule; the convention below is this build's - parity
 * against the paper's own system is unpinned for it):  cache bytes are OCP
 * FP8 E4M3 codes (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no
 * infinities, S.1111.111 = NaN, largest finite 448) in the same K token-major /
 * V dimension-major arrangement; a stored value stands for code_value * scale
 * with one float scale for K and one for V; the writer takes x / scale in
 * float32 (round to nearest) and rounds that to the nearest E4M3 value, ties to
 * the even code, magnitudes beyond 448 saturating to 448.  Attention over such a
 * cache is the same definition over the values the codes stand for.
 *
 * Parity pins live in tests/test_oracle_*.py (brute force, closed forms,
 * library cross-checks, the paper's worked examples).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 0, ORACLE_F32 = 1, ORACLE_FP8_E4M3 = 2 };

/* value of an E4M3 code: exponent field 0 is subnormal (m/8 * 2^-6), field 15 with mantissa 7 is NaN */
double oracle_e4m3_value(uint8_t code)
{
    int e = (code >> 3) & 15, m = code & 7;
    double mag;
    if (e == 15 && m == 7) return NAN;
    if (e == 0)
        mag = ldexp((double)m / 8.0, -6);
    else
        mag = ldexp(1.0 + (double)m / 8.0, e - 7);
    return (code & 0x80) ? -mag : mag;
}

/* nearest E4M3 code of a float: search the 127 finite magnitudes (codes 0x00..0x7e ascend with their
 * values), take the closer neighbour, the even code on a tie, 0x7e (448) beyond the range */
uint8_t oracle_e4m3_from_float(float f)
{
    uint8_t sign = signbit(f) ? 0x80 : 0x00;
    double a = fabs((double)f);
    int lo = 0;
    if (isnan(f)) return (uint8_t)(sign | 0x7f);
    if (a >= 448.0) return (uint8_t)(sign | 0x7e);
    while (lo < 0x7e && oracle_e4m3_value((uint8_t)(lo + 1)) <= a) ++lo; /* value(lo) <= a < value(lo+1) */
    {
        double below = a - oracle_e4m3_value((uint8_t)lo), above = oracle_e4m3_value((uint8_t)(lo + 1)) - a;
        int pick = lo;
        if (above < below || (above == below && (lo & 1))) pick = lo + 1;
        return (uint8_t)(sign | pick);
    }
}

static double widen(const void *base, size_t idx, int dtype)
{
    if (dtype == ORACLE_FP8_E4M3) return oracle_e4m3_value(((const uint8_t *)base)[idx]);
    if (dtype == ORACLE_BF16) {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return (double)((const float *)base)[idx];
}

static size_t esize_of(int dtype) { return dtype == ORACLE_BF16 ? 2 : (dtype == ORACLE_FP8_E4M3 ? 1 : 4); }

/* element index of K[token offset `off`][d] of KV head g in cache block `blk` */
static size_t k_elem(int64_t blk, int g, int off, int d, int hkv_l, int B, int D)
{
    return ((((size_t)blk * hkv_l + g) * 2 + 0) * (size_t)B + off) * D + d;
}

/* element index of V[d][token offset `off`] of KV head g in cache block `blk` */
static size_t v_elem(int64_t blk, int g, int off, int d, int hkv_l, int B, int D)
{
    return ((((size_t)blk * hkv_l + g) * 2 + 1) * (size_t)B * D) + (size_t)d * B + off;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------------------
 * Rank -> head block (Sec. 3.3.1).  TP groups are runs of consecutive global
 * ranks, SP groups take every TP-th rank.  A TP rank owns a contiguous column
 * slice of the heads; the SP exchange inside one SP group cuts that slice again
 * by SP rank.  So rank g = sp_rank*TP + tp_rank holds head block
 * tp_rank*SP + sp_rank.
 * ------------------------------------------------------------------------- */
int oracle_head_block(int sp, int tp, int rank)
{
    int tp_rank = rank % tp;
    int sp_rank = rank / tp;
    return tp_rank * sp + sp_rank;
}

/* KV head that destination `p` of a P-way exchange receives first: with h_kv
 * heads on the source, block p covers query heads [p*h/P, (p+1)*h/P) whose GQA
 * KV heads start at floor(p*h_kv/P) (Sec. 3.2.1, GQA extension / replication). */
int oracle_kv_head_of_block(int p, int P, int h_kv)
{
    return (int)(((int64_t)p * h_kv) / P);
}

/* ---------------------------------------------------------------------------
 * Send-side pack (Algorithm 1, first SP all-to-all).
 * in : qkv[T][h + 2*h_kv][D]     one fused row per token: q heads, k heads, v heads
 * out: send[P][T_pad][hq_l + 2*hkv_l][D], hq_l = h/P, hkv_l = max(1,h_kv/P)
 *      (h_kv == 0: query-only rows, hkv_l = 0).  Rows T..T_pad-1 are zero.
 * ------------------------------------------------------------------------- */
int oracle_pack_seq2head(const void *qkv, void *send, int T, int T_pad, int P, int h, int h_kv, int D,
                         int dtype)
{
    size_t e = esize_of(dtype), hb = (size_t)D * e; /* bytes of one head vector */
    int hq_l = h / P;
    int hkv_l = h_kv == 0 ? 0 : (h_kv >= P ? h_kv / P : 1);
    int w_in = h + 2 * h_kv, w_out = hq_l + 2 * hkv_l;
    const char *src = (const char *)qkv;
    char *dst = (char *)send;
    if (h % P) return -1;
    memset(dst, 0, (size_t)P * T_pad * w_out * hb);
    for (int p = 0; p < P; ++p) {
        int kv0 = h_kv ? oracle_kv_head_of_block(p, P, h_kv) : 0;
        for (int t = 0; t < T; ++t) {
            const char *row = src + (size_t)t * w_in * hb;
            char *orow = dst + ((size_t)p * T_pad + t) * w_out * hb;
            for (int j = 0; j < hq_l; ++j)
                memcpy(orow + (size_t)j * hb, row + (size_t)(p * hq_l + j) * hb, hb);
            for (int g = 0; g < hkv_l; ++g) {
                memcpy(orow + (size_t)(hq_l + g) * hb, row + (size_t)(h + kv0 + g) * hb, hb);
                memcpy(orow + (size_t)(hq_l + hkv_l + g) * hb, row + (size_t)(h + h_kv + kv0 + g) * hb, hb);
            }
        }
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Receive-side unpack (Algorithm 1, second SP all-to-all).
 * in : recv[P][T_pad][hq_l][D]  buffer p came from the rank holding head block p
 * out: out[T][h][D] with out[t][p*hq_l + j] = recv[p][t][j]; pad rows dropped.
 * ------------------------------------------------------------------------- */
int oracle_unpack_head2seq(const void *recv, void *out, int T, int T_pad, int P, int h, int D, int dtype)
{
    size_t hb = (size_t)D * esize_of(dtype);
    int hq_l = h / P;
    if (h % P) return -1;
    for (int p = 0; p < P; ++p)
        for (int t = 0; t < T; ++t)
            for (int j = 0; j < hq_l; ++j)
                memcpy((char *)out + ((size_t)t * h + p * hq_l + j) * hb,
                       (const char *)recv + (((size_t)p * T_pad + t) * hq_l + j) * hb, hb);
    return 0;
}

/* ---------------------------------------------------------------------------
 * KV-cache append (Sec. 2.2: prefill initialises the cache, each decoded token
 * is appended).  Token i of the batch goes to slot_mapping[i] = block*B + off;
 * a negative slot marks a padding row and writes nothing.
 * k_new, v_new: [n][hkv_l][D] dense.
 * ------------------------------------------------------------------------- */
int oracle_kv_write(const void *k_new, const void *v_new, const int64_t *slot_mapping, int64_t n,
                    void *kv_cache, int hkv_l, int D, int B, int dtype)
{
    size_t e = esize_of(dtype);
    for (int64_t i = 0; i < n; ++i) {
        int64_t slot = slot_mapping[i];
        if (slot < 0) continue;
        int64_t blk = slot / B;
        int off = (int)(slot % B);
        for (int g = 0; g < hkv_l; ++g)
            for (int d = 0; d < D; ++d) {
                size_t s = ((size_t)i * hkv_l + g) * D + d;
                memcpy((char *)kv_cache + k_elem(blk, g, off, d, hkv_l, B, D) * e, (const char *)k_new + s * e, e);
                memcpy((char *)kv_cache + v_elem(blk, g, off, d, hkv_l, B, D) * e, (const char *)v_new + s * e, e);
            }
    }
    return 0;
}

/* Append into an FP8 E4M3 cache: element x of k_new (stored in `src_dtype`) becomes the code nearest to
 * x / k_scale, the division taken in float32; v_new likewise with v_scale.  Same slots, same arrangement. */
int oracle_kv_write_fp8(const void *k_new, const void *v_new, const int64_t *slot_mapping, int64_t n,
                        void *kv_cache, int hkv_l, int D, int B, int src_dtype, float k_scale, float v_scale)
{
    uint8_t *c = (uint8_t *)kv_cache;
    if (!(k_scale > 0.0f) || !(v_scale > 0.0f)) return -1;
    for (int64_t i = 0; i < n; ++i) {
        int64_t slot = slot_mapping[i];
        if (slot < 0) continue;
        int64_t blk = slot / B;
        int off = (int)(slot % B);
        for (int g = 0; g < hkv_l; ++g)
            for (int d = 0; d < D; ++d) {
                size_t s = ((size_t)i * hkv_l + g) * D + d;
                float kx = (float)widen(k_new, s, src_dtype), vx = (float)widen(v_new, s, src_dtype);
                volatile float kq = kx / k_scale, vq = vx / v_scale; /* float32 quotients, not kept wider */
                c[k_elem(blk, g, off, d, hkv_l, B, D)] = oracle_e4m3_from_float(kq);
                c[v_elem(blk, g, off, d, hkv_l, B, D)] = oracle_e4m3_from_float(vq);
            }
    }
    return 0;
}

/* Rows of a matrix as FP8 E4M3 codes with one scale per row (the dynamic per-token scale of FP8
 * activations, and the per-output-feature scale of FP8 weights; Sec. 4.1 only says that FP8 models were
 * served, the rule is this build's reading): scale[r] = max_k |x[r][k]| / 448 as a float32 quotient
 * (1 for a row of zeros), code = the E4M3 code nearest to the float32 quotient x / scale[r].
 * x: [rows][cols] stored in `dtype`, row r starting at element r * row_stride. */
int oracle_quantize_rows_e4m3(const void *x, int dtype, int64_t rows, int64_t cols, int64_t row_stride,
                              uint8_t *codes, float *scales)
{
    if (dtype != ORACLE_BF16 && dtype != ORACLE_F32) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        float amax = 0.0f;
        for (int64_t k = 0; k < cols; ++k) {
            float a = fabsf((float)widen(x, (size_t)(r * row_stride + k), dtype));
            if (a > amax) amax = a;
        }
        volatile float sc = amax / 448.0f;
        float scale = amax > 0.0f ? sc : 1.0f;
        scales[r] = scale;
        for (int64_t k = 0; k < cols; ++k) {
            volatile float q = (float)widen(x, (size_t)(r * row_stride + k), dtype) / scale;
            codes[r * cols + k] = oracle_e4m3_from_float(q);
        }
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Attention of the local head shard over the paged cache (Algorithm 1, boxed
 * line; Sec. 2.2).  For sequence s with q_len new tokens out of ctx total,
 * new token i sits at position pos = ctx - q_len + i and sees keys 0..pos.
 * Query head j reads KV head j / (hq_l / hkv_l).
 *
 *   s_t  = scale * sum_d q[i][j][d] * K_s[t][g][d]          0 <= t <= pos
 *   p_t  = exp(s_t - max_t s_t) / sum_t exp(s_t - max_t s_t)
 *   out  = sum_t p_t * V_s[t][g][:]
 *
 * q   : [total_q][hq_l][D] stored in `dtype`
 * rows: optional list of query-token indices to evaluate (NULL: all of them);
 *       out is [n_rows][hq_l][D] doubles in the order of `rows`.
 * Returns 0, or -1 on inconsistent arguments.
 * ------------------------------------------------------------------------- */
int oracle_attention_kv(const void *q, int dtype, const void *kv_cache, int kv_dtype, double k_scale,
                        double v_scale, const int32_t *block_table, int max_blocks_per_seq,
                        const int32_t *cu_seqlens_q, const int32_t *seq_lens, int num_seqs, int hq_l, int hkv_l,
                        int D, int B, double scale, const int64_t *rows, int64_t n_rows, double *out);

/* cache stored in the same type as q, values as stored */
int oracle_attention(const void *q, const void *kv_cache, int dtype, const int32_t *block_table,
                     int max_blocks_per_seq, const int32_t *cu_seqlens_q, const int32_t *seq_lens,
                     int num_seqs, int hq_l, int hkv_l, int D, int B, double scale, const int64_t *rows,
                     int64_t n_rows, double *out)
{
    return oracle_attention_kv(q, dtype, kv_cache, dtype, 1.0, 1.0, block_table, max_blocks_per_seq, cu_seqlens_q,
                               seq_lens, num_seqs, hq_l, hkv_l, D, B, scale, rows, n_rows, out);
}

/* cache stored in `kv_dtype`; a stored K element stands for its value times k_scale, a V element for its
 * value times v_scale (both 1 for an unquantised cache) */
int oracle_attention_kv(const void *q, int dtype, const void *kv_cache, int kv_dtype, double k_scale,
                        double v_scale, const int32_t *block_table, int max_blocks_per_seq,
                        const int32_t *cu_seqlens_q, const int32_t *seq_lens, int num_seqs, int hq_l, int hkv_l,
                        int D, int B, double scale, const int64_t *rows, int64_t n_rows, double *out)
{
    int64_t total_q = num_seqs ? cu_seqlens_q[num_seqs] : 0;
    int group = hq_l / hkv_l;
    int bad = 0;
    if (hq_l % hkv_l) return -1;
    if (!rows) n_rows = total_q;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t item = 0; item < n_rows * hq_l; ++item) {
        int64_t r = item / hq_l;
        int j = (int)(item % hq_l);
        int64_t tok = rows ? rows[r] : r;
        int s = 0;
        if (tok < 0 || tok >= total_q) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        while (!(cu_seqlens_q[s] <= tok && tok < cu_seqlens_q[s + 1])) ++s;
        int q_len = cu_seqlens_q[s + 1] - cu_seqlens_q[s];
        int ctx = seq_lens[s];
        int i = (int)(tok - cu_seqlens_q[s]);
        int pos = ctx - q_len + i;
        int g = j / group;
        const int32_t *table = block_table + (size_t)s * max_blocks_per_seq;
        double *o = out + ((size_t)r * hq_l + j) * D;
        if (pos < 0 || ctx < q_len) {
#pragma omp atomic write
            bad = 1;
            continue;
        }

        double *logit = (double *)malloc((size_t)(pos + 1) * sizeof(double));
        double top = -INFINITY;
        for (int t = 0; t <= pos; ++t) {
            int64_t blk = table[t / B];
            double dot = 0.0;
            for (int d = 0; d < D; ++d)
                dot += widen(q, ((size_t)tok * hq_l + j) * D + d, dtype) *
                       (k_scale * widen(kv_cache, k_elem(blk, g, t % B, d, hkv_l, B, D), kv_dtype));
            logit[t] = scale * dot;
            if (logit[t] > top) top = logit[t];
        }
        double denom = 0.0;
        for (int t = 0; t <= pos; ++t) {
            logit[t] = exp(logit[t] - top);
            denom += logit[t];
        }
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int t = 0; t <= pos; ++t) {
            int64_t blk = table[t / B];
            double p = logit[t] / denom;
            for (int d = 0; d < D; ++d)
                o[d] += p * (v_scale * widen(kv_cache, v_elem(blk, g, t % B, d, hkv_l, B, D), kv_dtype));
        }
        free(logit);
    }
    return bad ? -1 : 0;
}
