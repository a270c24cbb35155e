// C-ABI front end: argument validation on the host, then kernel launches on the caller's stream.
// Nothing here allocates, frees, synchronises or reads device memory.
#include "../../include/shiftattn.h"
#include "../../include/shiftattn_probe.h"

#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

#include <atomic>
#include <mutex>

#include "internal.h"

using namespace shiftattn;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char* what) {
    return fail(SHIFTATTN_EHIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int elem_size(int dtype) { return dtype == SHIFTATTN_BF16 ? 2 : (dtype == SHIFTATTN_F32 ? 4 : 0); }

// process-wide tuning switches (shiftattn_set_option)
std::atomic<int> g_options[SHIFTATTN_OPT_COUNT];

bool force_generic() { return g_options[SHIFTATTN_OPT_GENERIC_ONLY].load(std::memory_order_relaxed) != 0; }

// Per-device set-up: three kernels need more dynamic LDS than a launch gets by default, which is an attribute of the
// function on each device.  Done once per device, under a lock, by the first call that may launch one of them there (or
// by shiftattn_init): safe from several host threads, and never inside a later call.
constexpr int kMaxDevices = 64;
std::mutex g_device_mu;
bool g_device_ready[kMaxDevices];

int ensure_device_ready() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(SHIFTATTN_EUNSUPPORTED, "device index %d: at most %d devices", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_device_mu);
    if (g_device_ready[dev]) return 0;
    if ((e = prefill_mfma_init()) != hipSuccess) return hip_fail(e, "set-up of the prefill kernel");
    if ((e = prefill_mfma64_init()) != hipSuccess) return hip_fail(e, "set-up of the wide prefill kernel");
    if ((e = proj_gemm_init()) != hipSuccess) return hip_fail(e, "set-up of the projection kernel");
    if ((e = proj_stream_init()) != hipSuccess) return hip_fail(e, "set-up of the small-batch projection kernel");
    g_device_ready[dev] = true;
    return 0;
}

// Fills `s` from the public struct; returns 0 or an error code.
int check_xchg(const shiftattn_xchg* x, int32_t T, int32_t T_pad, bool with_kv, XchgShape* s) {
    if (!x) return fail(SHIFTATTN_EINVAL, "exchange descriptor is NULL");
    const int e = elem_size(x->dtype);
    if (!e) return fail(SHIFTATTN_EINVAL, "unknown dtype %d", x->dtype);
    if (x->P < 1) return fail(SHIFTATTN_EINVAL, "P = %d must be >= 1", x->P);
    if (x->P > 1024) return fail(SHIFTATTN_EUNSUPPORTED, "P = %d: at most 1024 exchange members are supported", x->P);
    if (x->num_q_heads < 1 || x->num_q_heads % x->P)
        return fail(SHIFTATTN_EINVAL, "num_q_heads = %d must be a positive multiple of P = %d", x->num_q_heads, x->P);
    const int h_kv = with_kv ? x->num_kv_heads : 0;
    if (h_kv < 0) return fail(SHIFTATTN_EINVAL, "num_kv_heads = %d is negative", h_kv);
    if (h_kv > 0 && h_kv % x->P && x->P % h_kv)
        return fail(SHIFTATTN_EINVAL, "num_kv_heads = %d is neither a multiple nor a divisor of P = %d", h_kv, x->P);
    if (h_kv > 0 && x->num_q_heads % h_kv)
        return fail(SHIFTATTN_EINVAL, "num_q_heads = %d is not a multiple of num_kv_heads = %d", x->num_q_heads, h_kv);
    if (T < 0 || T_pad < T) return fail(SHIFTATTN_EINVAL, "need 0 <= T (%d) <= T_pad (%d)", T, T_pad);
    if (x->head_dim < 1) return fail(SHIFTATTN_EINVAL, "head_dim = %d", x->head_dim);
    if ((x->head_dim * e) % 16)
        return fail(SHIFTATTN_EUNSUPPORTED, "head_dim * element size = %d bytes is not a multiple of 16", x->head_dim * e);
    s->P = x->P;
    s->h = x->num_q_heads;
    s->h_kv = h_kv;
    s->hq_l = x->num_q_heads / x->P;
    s->hkv_l = h_kv == 0 ? 0 : (h_kv >= x->P ? h_kv / x->P : 1);
    if (h_kv > 0) {
        // the q heads of one destination must sit inside the GQA groups of the KV heads it receives
        const int group = x->num_q_heads / h_kv;
        if (s->hq_l % group && group % s->hq_l)
            return fail(SHIFTATTN_EINVAL, "h/P = %d neither divides nor is a multiple of the GQA group h/h_kv = %d",
                        s->hq_l, group);
    }
    s->vec_per_head = x->head_dim * e / 16;
    s->T = T;
    s->T_pad = T_pad;
    const uint64_t in_vecs = static_cast<uint64_t>(T) * (s->h + 2 * s->h_kv) * s->vec_per_head;
    const uint64_t out_vecs = static_cast<uint64_t>(T_pad) * (s->hq_l + 2 * s->hkv_l) * s->vec_per_head;
    if (in_vecs > 0x7FFFFFFFull || out_vecs > 0x7FFFFFFFull)
        return fail(SHIFTATTN_EUNSUPPORTED, "more than 2^31-1 16-byte vectors per buffer");
    return 0;
}

int check_attn(const shiftattn_attn* a, AttnShape* s) {
    if (!a) return fail(SHIFTATTN_EINVAL, "attention descriptor is NULL");
    const int e = elem_size(a->dtype);
    if (!e) return fail(SHIFTATTN_EINVAL, "unknown dtype %d", a->dtype);
    if (a->num_q_heads < 1 || a->num_kv_heads < 1 || a->num_q_heads % a->num_kv_heads)
        return fail(SHIFTATTN_EINVAL, "num_q_heads = %d must be a positive multiple of num_kv_heads = %d",
                    a->num_q_heads, a->num_kv_heads);
    if (a->head_dim < 1) return fail(SHIFTATTN_EINVAL, "head_dim = %d", a->head_dim);
    if (a->head_dim % 8 || a->head_dim > 256)
        return fail(SHIFTATTN_EUNSUPPORTED, "head_dim = %d: need a multiple of 8 up to 256", a->head_dim);
    if (a->block_size != kBlockSize) return fail(SHIFTATTN_EUNSUPPORTED, "block_size = %d: only 16 is built", a->block_size);
    if (a->num_blocks < 0 || a->max_blocks_per_seq < 0)
        return fail(SHIFTATTN_EINVAL, "num_blocks = %d, max_blocks_per_seq = %d", a->num_blocks, a->max_blocks_per_seq);
    if (!(a->softmax_scale > 0.f) || a->softmax_scale > 3.0e38f)
        return fail(SHIFTATTN_EINVAL, "softmax_scale must be positive and finite");
    s->hq_l = a->num_q_heads;
    s->hkv_l = a->num_kv_heads;
    s->D = a->head_dim;
    s->elem = e;
    s->num_blocks = a->num_blocks;
    s->max_blocks = a->max_blocks_per_seq;
    s->scale = a->softmax_scale;
    s->q_stride = a->q_stride ? a->q_stride : static_cast<int64_t>(s->hq_l) * s->D;
    s->kv_stride = a->kv_stride ? a->kv_stride : static_cast<int64_t>(s->hkv_l) * s->D;
    s->out_stride = a->out_stride ? a->out_stride : static_cast<int64_t>(s->hq_l) * s->D;
    if (s->q_stride < static_cast<int64_t>(s->hq_l) * s->D || s->out_stride < static_cast<int64_t>(s->hq_l) * s->D ||
        s->kv_stride < static_cast<int64_t>(s->hkv_l) * s->D)
        return fail(SHIFTATTN_EINVAL, "a row stride is smaller than the row it strides over");
    if ((s->q_stride * e) % 16 || (s->kv_stride * e) % 16 || (s->out_stride * e) % 16)
        return fail(SHIFTATTN_EINVAL, "row strides must be multiples of 16 bytes");
    s->kv_elem = e;
    s->k_scale = s->v_scale = 1.f;
    if (a->kv_format == SHIFTATTN_KV_FP8_E4M3) {
        if (!(a->k_scale > 0.f) || !(a->v_scale > 0.f) || a->k_scale > 3.0e38f || a->v_scale > 3.0e38f)
            return fail(SHIFTATTN_EINVAL, "k_scale and v_scale of an FP8 cache must be positive and finite");
        if (a->head_dim % 16) return fail(SHIFTATTN_EUNSUPPORTED, "head_dim = %d: an FP8 cache needs a multiple of 16", a->head_dim);
        s->kv_elem = 1;
        s->k_scale = a->k_scale;
        s->v_scale = a->v_scale;
    } else if (a->kv_format != SHIFTATTN_KV_SAME) {
        return fail(SHIFTATTN_EINVAL, "unknown kv_format %d", a->kv_format);
    }
    if (a->reserved != 0) return fail(SHIFTATTN_EINVAL, "reserved field must be 0");
    return 0;
}

int check_new_kv(const void* k_new, const void* v_new, const int64_t* slots, bool* present) {
    const int n = (k_new != nullptr) + (v_new != nullptr) + (slots != nullptr);
    if (n != 0 && n != 3) return fail(SHIFTATTN_EINVAL, "k_new, v_new and slot_mapping must be all NULL or all set");
    if (n == 3 && (!aligned16(k_new) || !aligned16(v_new)))
        return fail(SHIFTATTN_EINVAL, "k_new / v_new must be 16-byte aligned");
    *present = n == 3;
    return 0;
}

bool use_prefill_mfma(const AttnShape& s, int num_seqs, int max_seq_len) {
    return !force_generic() && prefill_mfma_supported(s, num_seqs, max_seq_len);
}
bool use_decode_mfma(const AttnShape& s, int num_seqs, int max_seq_len) {
    return !force_generic() && decode_mfma_supported(s, num_seqs, max_seq_len);
}

// Argument checks of a prefill / decode call that need no launch (shared with the mixed entry point, which must
// not have written the cache when one of them fails).
int check_prefill_args(const void* q, const void* kv_cache, const int32_t* block_table, const int32_t* cu_seqlens_q,
                       const int32_t* seq_lens, int32_t num_seqs, int32_t total_q, int32_t max_q_len, int32_t max_seq_len,
                       const void* out, const AttnShape& s) {
    if (num_seqs < 0 || total_q < 0 || max_q_len < 0 || max_seq_len < 0)
        return fail(SHIFTATTN_EINVAL, "negative size argument");
    if (max_q_len > total_q || max_q_len > max_seq_len)
        return fail(SHIFTATTN_EINVAL, "max_q_len = %d exceeds total_q = %d or max_seq_len = %d", max_q_len, total_q,
                    max_seq_len);
    if (num_seqs == 0 || total_q == 0) return 0;
    if (!q || !kv_cache || !block_table || !cu_seqlens_q || !seq_lens || !out)
        return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(q) || !aligned16(out) || !aligned16(kv_cache))
        return fail(SHIFTATTN_EINVAL, "q / out / kv_cache must be 16-byte aligned");
    if (static_cast<int64_t>(s.max_blocks) * kBlockSize < max_seq_len)
        return fail(SHIFTATTN_EINVAL, "max_blocks_per_seq = %d cannot hold max_seq_len = %d", s.max_blocks, max_seq_len);
    return 0;
}

int check_decode_args(const void* q, const void* kv_cache, const int32_t* block_table, const int32_t* seq_lens,
                      int32_t num_seqs, int32_t max_seq_len, const void* out, const AttnShape& s) {
    if (num_seqs < 0 || max_seq_len < 0) return fail(SHIFTATTN_EINVAL, "negative size argument");
    if (num_seqs == 0) return 0;
    if (!q || !kv_cache || !block_table || !seq_lens || !out) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(q) || !aligned16(out) || !aligned16(kv_cache))
        return fail(SHIFTATTN_EINVAL, "q / out / kv_cache must be 16-byte aligned");
    if (static_cast<int64_t>(s.max_blocks) * kBlockSize < max_seq_len)
        return fail(SHIFTATTN_EINVAL, "max_blocks_per_seq = %d cannot hold max_seq_len = %d", s.max_blocks, max_seq_len);
    return 0;
}

// ---- device memory the library itself holds, for shiftattn_decode_static -------------------------------------
// One array per GPU the library runs on, held until the process ends.  In host code the array's name is only a
// handle: its device address is looked up once per device (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[SHIFTATTN_STATIC_SCRATCH_BYTES];

std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];  // per device: address of `scratch` there, null until first looked up

int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(SHIFTATTN_EUNSUPPORTED, "device index %d: at most %d devices", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!ptr) return fail(SHIFTATTN_EHIP, "hipGetSymbolAddress(scratch) returned a null address");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return 0;
}

}  // namespace

namespace shiftattn {
int option_prefill_tile() { return g_options[SHIFTATTN_OPT_PREFILL_TILE].load(std::memory_order_relaxed); }
int option_prefill_splits() { return g_options[SHIFTATTN_OPT_PREFILL_SPLITS].load(std::memory_order_relaxed); }
int option_prefill_pairing() { return g_options[SHIFTATTN_OPT_PREFILL_PAIRING].load(std::memory_order_relaxed); }
int option_prefill_scaled_q() { return g_options[SHIFTATTN_OPT_PREFILL_SCALED_Q].load(std::memory_order_relaxed); }
}  // namespace shiftattn

extern "C" {

const char* shiftattn_last_error(void) { return g_err; }

int shiftattn_init(void) {
    if (int rc = ensure_device_ready()) return rc;
    void* ws = nullptr;
    return static_scratch(&ws);
}

int shiftattn_set_option(int32_t option, int32_t value) {
    switch (option) {
        case SHIFTATTN_OPT_PREFILL_TILE:
            if (value != 0 && value != 128 && value != 256)
                return fail(SHIFTATTN_EINVAL, "SHIFTATTN_OPT_PREFILL_TILE takes 0, 128 or 256, not %d", value);
            break;
        case SHIFTATTN_OPT_PREFILL_SPLITS:
            if (value < 0 || value > 64) return fail(SHIFTATTN_EINVAL, "SHIFTATTN_OPT_PREFILL_SPLITS takes 0 .. 64, not %d", value);
            break;
        case SHIFTATTN_OPT_GENERIC_ONLY:
            if (value != 0 && value != 1) return fail(SHIFTATTN_EINVAL, "SHIFTATTN_OPT_GENERIC_ONLY takes 0 or 1, not %d", value);
            break;
        case SHIFTATTN_OPT_PREFILL_PAIRING:
            if (value < 0 || value > 2) return fail(SHIFTATTN_EINVAL, "SHIFTATTN_OPT_PREFILL_PAIRING takes 0, 1 or 2, not %d", value);
            break;
        case SHIFTATTN_OPT_PREFILL_SCALED_Q:
            if (value != 0 && value != 1) return fail(SHIFTATTN_EINVAL, "SHIFTATTN_OPT_PREFILL_SCALED_Q takes 0 or 1, not %d", value);
            break;
        default:
            return fail(SHIFTATTN_EINVAL, "unknown option %d", option);
    }
    g_options[option].store(value, std::memory_order_relaxed);
    return SHIFTATTN_OK;
}

int32_t shiftattn_get_option(int32_t option) {
    if (option < 0 || option >= SHIFTATTN_OPT_COUNT) return -1;
    return g_options[option].load(std::memory_order_relaxed);
}

int32_t shiftattn_head_block(int32_t sp, int32_t tp, int32_t rank) {
    if (sp < 1 || tp < 1 || rank < 0 || rank >= sp * tp) return -1;
    return (rank % tp) * sp + rank / tp;
}

int32_t shiftattn_kv_head_of_block(int32_t block, int32_t P, int32_t h_kv) {
    if (P < 1 || h_kv < 1 || block < 0 || block >= P) return -1;
    return static_cast<int32_t>((static_cast<int64_t>(block) * h_kv) / P);
}

int32_t shiftattn_padded_tokens(int32_t n, int32_t sp) {
    if (n < 0 || sp < 1) return -1;
    const int64_t padded = (static_cast<int64_t>(n) + sp - 1) / sp * sp;
    return padded > 0x7FFFFFFF ? -1 : static_cast<int32_t>(padded);
}

int32_t shiftattn_use_base_config(int32_t n_tokens, int32_t threshold) {
    if (n_tokens < 0 || threshold < 0) return -1;
    return n_tokens > threshold ? 1 : 0;
}

int shiftattn_ceiling_mfma_bf16(const void* operands, void* sink, int32_t iters, int64_t* flops, void* stream) {
    if (!operands || !sink || !flops) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(operands)) return fail(SHIFTATTN_EINVAL, "operands must be 16-byte aligned");
    if (iters < 1 || iters > (1 << 24)) return fail(SHIFTATTN_EINVAL, "iters = %d", iters);
    hipError_t e = launch_mfma_ceiling(operands, sink, iters, flops, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "ceiling_mfma launch");
}

int shiftattn_ceiling_mfma_bf16_fresh(const void* operands, void* sink, int32_t iters, int64_t* flops, void* stream) {
    if (!operands || !sink || !flops) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(operands)) return fail(SHIFTATTN_EINVAL, "operands must be 16-byte aligned");
    if (iters < 1 || iters > (1 << 24)) return fail(SHIFTATTN_EINVAL, "iters = %d", iters);
    hipError_t e = launch_mfma_ceiling_fresh(operands, sink, iters, flops, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "ceiling_mfma_fresh launch");
}

int shiftattn_ceiling_hbm_read(const void* src, size_t bytes, void* sink, int64_t* bytes_read, void* stream) {
    if (!src || !sink || !bytes_read) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(src)) return fail(SHIFTATTN_EINVAL, "src must be 16-byte aligned");
    hipError_t e = launch_hbm_read_ceiling(src, bytes, sink, bytes_read, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "ceiling_hbm_read launch");
}

int shiftattn_ceiling_hbm_copy(const void* src, void* dst, size_t bytes, int64_t* bytes_copied, void* stream) {
    if (!src || !dst || !bytes_copied) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(src) || !aligned16(dst)) return fail(SHIFTATTN_EINVAL, "src / dst must be 16-byte aligned");
    hipError_t e = launch_hbm_copy_ceiling(src, dst, bytes, bytes_copied, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "ceiling_hbm_copy launch");
}

int shiftattn_pack_seq2head(const void* qkv, void* send, int32_t T, int32_t T_pad, const shiftattn_xchg* x,
                            void* stream) {
    XchgShape s;
    if (int rc = check_xchg(x, T, T_pad, true, &s)) return rc;
    if (T_pad == 0) return SHIFTATTN_OK;
    if (!send || (T > 0 && !qkv)) return fail(SHIFTATTN_EINVAL, "qkv or send is NULL");
    if (!aligned16(qkv) || !aligned16(send)) return fail(SHIFTATTN_EINVAL, "qkv / send must be 16-byte aligned");
    hipError_t e = launch_pack(qkv, send, s, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "pack_seq2head launch");
}

int shiftattn_unpack_head2seq(const void* recv, void* out, int32_t T, int32_t T_pad, const shiftattn_xchg* x,
                              void* stream) {
    XchgShape s;
    if (int rc = check_xchg(x, T, T_pad, false, &s)) return rc;
    if (T == 0) return SHIFTATTN_OK;
    if (!recv || !out) return fail(SHIFTATTN_EINVAL, "recv or out is NULL");
    if (!aligned16(recv) || !aligned16(out)) return fail(SHIFTATTN_EINVAL, "recv / out must be 16-byte aligned");
    hipError_t e = launch_unpack(recv, out, s, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "unpack_head2seq launch");
}

int shiftattn_qkv_proj_pack_ws(const void* x, const void* w_qkv, void* send, int32_t T, int32_t T_pad, int32_t d_model,
                               const shiftattn_xchg* xc, void* workspace, size_t workspace_bytes, void* stream) {
    XchgShape s;
    if (int rc = check_xchg(xc, T, T_pad, true, &s)) return rc;
    if (d_model < 1) return fail(SHIFTATTN_EINVAL, "d_model = %d", d_model);
    if (!qkv_proj_pack_supported(s, d_model, elem_size(xc->dtype)))
        return fail(SHIFTATTN_EUNSUPPORTED, "projection into the send buffers is built for bf16, head_dim 128, d_model a multiple "
                                            "of 64 and an even number of heads per row (got d_model = %d, %d heads)",
                    d_model, s.h + 2 * s.h_kv);
    if (s.T_pad == 0) return SHIFTATTN_OK;
    if (!send || (s.T > 0 && (!x || !w_qkv))) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(x) || !aligned16(w_qkv) || !aligned16(send)) return fail(SHIFTATTN_EINVAL, "x / w_qkv / send must be 16-byte aligned");
    if (workspace_bytes > 0 && (!workspace || !aligned16(workspace)))
        return fail(SHIFTATTN_EINVAL, "workspace is NULL or not 16-byte aligned");
    if (int rc = ensure_device_ready()) return rc;
    const int n_feat = (s.h + 2 * s.h_kv) * 128;
    hipError_t e;
    if (s.T > 0 && !force_generic() && proj_stream_takes(s.T_pad, n_feat, d_model, false, workspace_bytes))
        e = launch_qkv_proj_stream(x, w_qkv, send, d_model, s, nullptr, nullptr, workspace, static_cast<hipStream_t>(stream));
    else
        e = launch_qkv_proj_pack(x, w_qkv, send, d_model, s, nullptr, nullptr, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "qkv_proj_pack launch");
}

int shiftattn_qkv_proj_pack(const void* x, const void* w_qkv, void* send, int32_t T, int32_t T_pad, int32_t d_model,
                            const shiftattn_xchg* xc, void* stream) {
    return shiftattn_qkv_proj_pack_ws(x, w_qkv, send, T, T_pad, d_model, xc, nullptr, 0, stream);
}

int shiftattn_unpack_o_proj_ws(const void* recv, const void* w_o, void* out, int32_t T, int32_t T_pad, int32_t d_model,
                               const shiftattn_xchg* xc, void* workspace, size_t workspace_bytes, void* stream) {
    XchgShape s;
    if (int rc = check_xchg(xc, T, T_pad, false, &s)) return rc;
    if (d_model < 1) return fail(SHIFTATTN_EINVAL, "d_model = %d", d_model);
    if (!unpack_o_proj_supported(s, d_model, elem_size(xc->dtype)))
        return fail(SHIFTATTN_EUNSUPPORTED, "projection out of the receive buffers is built for bf16, head_dim 128 and d_model a "
                                            "multiple of 256 (got d_model = %d)", d_model);
    if (s.T == 0) return SHIFTATTN_OK;
    if (!recv || !w_o || !out) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(recv) || !aligned16(w_o) || !aligned16(out)) return fail(SHIFTATTN_EINVAL, "recv / w_o / out must be 16-byte aligned");
    if (workspace_bytes > 0 && (!workspace || !aligned16(workspace)))
        return fail(SHIFTATTN_EINVAL, "workspace is NULL or not 16-byte aligned");
    if (int rc = ensure_device_ready()) return rc;
    hipError_t e;
    if (!force_generic() && proj_stream_takes(s.T, d_model, s.h * 128, false, workspace_bytes))
        e = launch_o_proj_stream(recv, w_o, out, d_model, s, nullptr, nullptr, workspace, static_cast<hipStream_t>(stream));
    else
        e = launch_unpack_o_proj(recv, w_o, out, d_model, s, nullptr, nullptr, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "unpack_o_proj launch");
}

int shiftattn_unpack_o_proj(const void* recv, const void* w_o, void* out, int32_t T, int32_t T_pad, int32_t d_model,
                            const shiftattn_xchg* xc, void* stream) {
    return shiftattn_unpack_o_proj_ws(recv, w_o, out, T, T_pad, d_model, xc, nullptr, 0, stream);
}

size_t shiftattn_proj_workspace_bytes(int32_t rows, int32_t n_features, int32_t k) {
    if (rows < 1 || n_features < 1 || k < 1 || force_generic()) return 0;
    if (proj_stream_takes(rows, n_features, k, false, static_cast<size_t>(-1))) return proj_stream_workspace(rows, n_features, k, false);
    return proj_gemm_workspace(rows, n_features, k, false);
}

size_t shiftattn_proj_workspace_bytes_fp8(int32_t rows, int32_t n_features, int32_t k) {
    if (rows < 1 || n_features < 1 || k < 1 || force_generic()) return 0;
    if (proj_stream_takes(rows, n_features, k, true, static_cast<size_t>(-1))) return proj_stream_workspace(rows, n_features, k, true);
    return proj_gemm_workspace(rows, n_features, k, true);
}

int shiftattn_quantize_rows_fp8(const void* x, void* codes, float* scales, int32_t rows, int32_t cols, void* stream) {
    if (rows < 0 || cols < 1) return fail(SHIFTATTN_EINVAL, "rows = %d, cols = %d", rows, cols);
    if (cols % 8) return fail(SHIFTATTN_EUNSUPPORTED, "cols = %d is not a multiple of 8", cols);
    if (rows == 0) return SHIFTATTN_OK;
    if (!x || !codes || !scales) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(codes) & 7) || (reinterpret_cast<uintptr_t>(scales) & 3))
        return fail(SHIFTATTN_EINVAL, "x must be 16-byte, codes 8-byte, scales 4-byte aligned");
    hipError_t e = launch_quantize_rows_fp8(x, codes, scales, rows, cols, cols, 0, cols, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "quantize_rows_fp8 launch");
}

int shiftattn_quantize_recv_fp8(const void* recv, void* codes, float* scales, int32_t T, int32_t T_pad,
                                const shiftattn_xchg* xc, void* stream) {
    XchgShape s;
    if (int rc = check_xchg(xc, T, T_pad, false, &s)) return rc;
    if (xc->dtype != SHIFTATTN_BF16) return fail(SHIFTATTN_EUNSUPPORTED, "the quantiser reads bf16 rows");
    if (xc->head_dim % 8) return fail(SHIFTATTN_EUNSUPPORTED, "head_dim = %d is not a multiple of 8", xc->head_dim);
    if (s.T == 0) return SHIFTATTN_OK;
    if (!recv || !codes || !scales) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(recv) || (reinterpret_cast<uintptr_t>(codes) & 7) || (reinterpret_cast<uintptr_t>(scales) & 3))
        return fail(SHIFTATTN_EINVAL, "recv must be 16-byte, codes 8-byte, scales 4-byte aligned");
    const int seg = s.hq_l * xc->head_dim;
    hipError_t e = launch_quantize_rows_fp8(recv, codes, scales, s.T, s.P * seg, seg, static_cast<int64_t>(s.T_pad) * seg, seg,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "quantize_recv_fp8 launch");
}

int shiftattn_qkv_proj_pack_fp8_ws(const void* x_codes, const float* x_scales, const void* w_codes, const float* w_scales,
                                   void* send, int32_t T, int32_t T_pad, int32_t d_model, const shiftattn_xchg* xc,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    XchgShape s;
    if (int rc = check_xchg(xc, T, T_pad, true, &s)) return rc;
    if (d_model < 1) return fail(SHIFTATTN_EINVAL, "d_model = %d", d_model);
    if (!qkv_proj_pack_supported(s, d_model, elem_size(xc->dtype)))
        return fail(SHIFTATTN_EUNSUPPORTED, "projection into the send buffers is built for bf16 results, head_dim 128, d_model a "
                                            "multiple of 64 and an even number of heads per row (got d_model = %d, %d heads)",
                    d_model, s.h + 2 * s.h_kv);
    if (s.T_pad == 0) return SHIFTATTN_OK;
    if (!send || (s.T > 0 && (!x_codes || !w_codes || !x_scales || !w_scales))) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(x_codes) || !aligned16(w_codes) || !aligned16(send) || !aligned16(w_scales) || (reinterpret_cast<uintptr_t>(x_scales) & 3))
        return fail(SHIFTATTN_EINVAL, "x_codes / w_codes / w_scales / send must be 16-byte aligned, x_scales 4-byte");
    if (workspace_bytes > 0 && (!workspace || !aligned16(workspace)))
        return fail(SHIFTATTN_EINVAL, "workspace is NULL or not 16-byte aligned");
    if (int rc = ensure_device_ready()) return rc;
    const int n_feat = (s.h + 2 * s.h_kv) * 128;
    hipError_t e;
    if (s.T > 0 && !force_generic() && proj_stream_takes(s.T_pad, n_feat, d_model, true, workspace_bytes))
        e = launch_qkv_proj_stream(x_codes, w_codes, send, d_model, s, x_scales, w_scales, workspace, static_cast<hipStream_t>(stream));
    else
        e = launch_qkv_proj_pack(x_codes, w_codes, send, d_model, s, x_scales, w_scales, force_generic() ? nullptr : workspace,
                                 workspace_bytes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "qkv_proj_pack_fp8 launch");
}

int shiftattn_qkv_proj_pack_fp8(const void* x_codes, const float* x_scales, const void* w_codes, const float* w_scales,
                                void* send, int32_t T, int32_t T_pad, int32_t d_model, const shiftattn_xchg* xc, void* stream) {
    return shiftattn_qkv_proj_pack_fp8_ws(x_codes, x_scales, w_codes, w_scales, send, T, T_pad, d_model, xc, nullptr, 0, stream);
}

int shiftattn_unpack_o_proj_fp8_ws(const void* recv_codes, const float* a_scales, const void* w_codes, const float* w_scales,
                                   void* out, int32_t T, int32_t T_pad, int32_t d_model, const shiftattn_xchg* xc,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    XchgShape s;
    if (int rc = check_xchg(xc, T, T_pad, false, &s)) return rc;
    if (d_model < 1) return fail(SHIFTATTN_EINVAL, "d_model = %d", d_model);
    if (!unpack_o_proj_supported(s, d_model, elem_size(xc->dtype)))
        return fail(SHIFTATTN_EUNSUPPORTED, "projection out of the receive buffers is built for bf16 results, head_dim 128 and "
                                            "d_model a multiple of 256 (got d_model = %d)", d_model);
    if (s.T == 0) return SHIFTATTN_OK;
    if (!recv_codes || !a_scales || !w_codes || !w_scales || !out) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(recv_codes) || !aligned16(w_codes) || !aligned16(out) || !aligned16(w_scales) || (reinterpret_cast<uintptr_t>(a_scales) & 3))
        return fail(SHIFTATTN_EINVAL, "recv_codes / w_codes / w_scales / out must be 16-byte aligned, a_scales 4-byte");
    if (workspace_bytes > 0 && (!workspace || !aligned16(workspace)))
        return fail(SHIFTATTN_EINVAL, "workspace is NULL or not 16-byte aligned");
    if (int rc = ensure_device_ready()) return rc;
    hipError_t e;
    if (!force_generic() && proj_stream_takes(s.T, d_model, s.h * 128, true, workspace_bytes))
        e = launch_o_proj_stream(recv_codes, w_codes, out, d_model, s, a_scales, w_scales, workspace, static_cast<hipStream_t>(stream));
    else
        e = launch_unpack_o_proj(recv_codes, w_codes, out, d_model, s, a_scales, w_scales, force_generic() ? nullptr : workspace,
                                 workspace_bytes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "unpack_o_proj_fp8 launch");
}

int shiftattn_unpack_o_proj_fp8(const void* recv_codes, const float* a_scales, const void* w_codes, const float* w_scales,
                                void* out, int32_t T, int32_t T_pad, int32_t d_model, const shiftattn_xchg* xc, void* stream) {
    return shiftattn_unpack_o_proj_fp8_ws(recv_codes, a_scales, w_codes, w_scales, out, T, T_pad, d_model, xc, nullptr, 0, stream);
}

int shiftattn_kv_write(const void* k_new, const void* v_new, const int64_t* slot_mapping, int32_t n_tokens,
                       void* kv_cache, const shiftattn_attn* a, void* stream) {
    AttnShape s;
    if (int rc = check_attn(a, &s)) return rc;
    if (n_tokens < 0) return fail(SHIFTATTN_EINVAL, "n_tokens = %d", n_tokens);
    if (n_tokens == 0) return SHIFTATTN_OK;
    if (!k_new || !v_new || !slot_mapping || !kv_cache) return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(kv_cache))
        return fail(SHIFTATTN_EINVAL, "k_new / v_new / kv_cache must be 16-byte aligned");
    hipError_t e = launch_kv_write(k_new, v_new, slot_mapping, n_tokens, kv_cache, s, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "kv_write launch");
}

size_t shiftattn_prefill_workspace_bytes(int32_t num_seqs, int32_t total_q, int32_t max_q_len, int32_t max_seq_len,
                                         const shiftattn_attn* a) {
    AttnShape s;
    if (check_attn(a, &s) || num_seqs < 0 || total_q < 0 || max_q_len < 0 || max_seq_len < 0) return SIZE_MAX;
    if (!use_prefill_mfma(s, num_seqs, max_seq_len) || num_seqs == 0 || total_q == 0) return 0;
    return prefill_mfma_workspace(num_seqs, total_q, max_q_len, max_seq_len, s);
}

size_t shiftattn_decode_workspace_bytes(int32_t num_seqs, int32_t max_seq_len, const shiftattn_attn* a) {
    AttnShape s;
    if (check_attn(a, &s) || num_seqs < 0 || max_seq_len < 0) return SIZE_MAX;
    if (!use_decode_mfma(s, num_seqs, max_seq_len) || num_seqs == 0) return 0;
    return decode_mfma_workspace(num_seqs, max_seq_len, s);
}

int shiftattn_prefill(const void* q, const void* k_new, const void* v_new, const int64_t* slot_mapping, void* kv_cache,
                      const int32_t* block_table, const int32_t* cu_seqlens_q, const int32_t* seq_lens,
                      int32_t num_seqs, int32_t total_q, int32_t max_q_len, int32_t max_seq_len, void* out,
                      void* workspace, size_t workspace_bytes, const shiftattn_attn* a, void* stream) {
    AttnShape s;
    if (int rc = check_attn(a, &s)) return rc;
    bool new_kv;
    if (int rc = check_new_kv(k_new, v_new, slot_mapping, &new_kv)) return rc;
    if (int rc = check_prefill_args(q, kv_cache, block_table, cu_seqlens_q, seq_lens, num_seqs, total_q, max_q_len,
                                    max_seq_len, out, s))
        return rc;
    if (num_seqs == 0 || total_q == 0) return SHIFTATTN_OK;
    const bool mfma = use_prefill_mfma(s, num_seqs, max_seq_len);
    const size_t need = mfma ? prefill_mfma_workspace(num_seqs, total_q, max_q_len, max_seq_len, s) : 0;
    if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace)))
        return fail(SHIFTATTN_EWORKSPACE, "prefill needs %zu workspace bytes, got %zu", need,
                    workspace ? workspace_bytes : static_cast<size_t>(0));
    if (mfma)
        if (int rc = ensure_device_ready()) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (new_kv) {
        e = launch_kv_write(k_new, v_new, slot_mapping, total_q, kv_cache, s, st);
        if (e != hipSuccess) return hip_fail(e, "kv_write launch");
    }
    if (mfma)
        e = launch_prefill_mfma(q, kv_cache, block_table, cu_seqlens_q, seq_lens, num_seqs, total_q, max_q_len,
                                max_seq_len, out, workspace, s, st);
    else
        e = launch_attn_generic(q, kv_cache, block_table, cu_seqlens_q, seq_lens, num_seqs, total_q, out, s, st);
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "prefill launch");
}

int shiftattn_decode(const void* q, const void* k_new, const void* v_new, const int64_t* slot_mapping, void* kv_cache,
                     const int32_t* block_table, const int32_t* seq_lens, int32_t num_seqs, int32_t max_seq_len,
                     void* out, void* workspace, size_t workspace_bytes, const shiftattn_attn* a, void* stream) {
    AttnShape s;
    if (int rc = check_attn(a, &s)) return rc;
    bool new_kv;
    if (int rc = check_new_kv(k_new, v_new, slot_mapping, &new_kv)) return rc;
    if (int rc = check_decode_args(q, kv_cache, block_table, seq_lens, num_seqs, max_seq_len, out, s)) return rc;
    if (num_seqs == 0) return SHIFTATTN_OK;
    const bool mfma = use_decode_mfma(s, num_seqs, max_seq_len);
    const size_t need = mfma ? decode_mfma_workspace(num_seqs, max_seq_len, s) : 0;
    if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace)))
        return fail(SHIFTATTN_EWORKSPACE, "decode needs %zu workspace bytes, got %zu", need,
                    workspace ? workspace_bytes : static_cast<size_t>(0));
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    // the tuned kernel appends the new tokens itself where it can; otherwise a write kernel runs in front
    const bool fused_append = new_kv && mfma && decode_mfma_appends(num_seqs, s);
    if (new_kv && !fused_append) {
        e = launch_kv_write(k_new, v_new, slot_mapping, num_seqs, kv_cache, s, st);
        if (e != hipSuccess) return hip_fail(e, "kv_write launch");
    }
    if (mfma)
        e = launch_decode_mfma(q, fused_append ? k_new : nullptr, fused_append ? v_new : nullptr,
                               fused_append ? slot_mapping : nullptr, kv_cache, block_table, seq_lens, num_seqs, max_seq_len,
                               out, workspace, s, st);
    else
        e = launch_attn_generic(q, kv_cache, block_table, nullptr, seq_lens, num_seqs, num_seqs, out, s, st);
    return e == hipSuccess ? SHIFTATTN_OK : hip_fail(e, "decode launch");
}

int shiftattn_decode_static(const void* q, const void* k_new, const void* v_new, const int64_t* slot_mapping, void* kv_cache,
                            const int32_t* block_table, const int32_t* seq_lens, int32_t num_seqs, int32_t max_seq_len,
                            void* out, const shiftattn_attn* a, void* stream) {
    const size_t need = shiftattn_decode_workspace_bytes(num_seqs, max_seq_len, a);
    if (need == SIZE_MAX) {  // let the ordinary entry point name the bad argument (it needs no workspace to do so)
        return shiftattn_decode(q, k_new, v_new, slot_mapping, kv_cache, block_table, seq_lens, num_seqs, max_seq_len, out,
                                nullptr, 0, a, stream);
    }
    if (need > SHIFTATTN_STATIC_SCRATCH_BYTES)
        return fail(SHIFTATTN_EWORKSPACE,
                    "decode_static: this batch needs %zu bytes of split partials, the library's own scratch holds %zu; "
                    "use shiftattn_decode with a caller-provided workspace",
                    need, static_cast<size_t>(SHIFTATTN_STATIC_SCRATCH_BYTES));
    void* ws = nullptr;
    if (need > 0)
        if (int rc = static_scratch(&ws)) return rc;
    return shiftattn_decode(q, k_new, v_new, slot_mapping, kv_cache, block_table, seq_lens, num_seqs, max_seq_len, out, ws,
                            need > 0 ? static_cast<size_t>(SHIFTATTN_STATIC_SCRATCH_BYTES) : 0, a, stream);
}

size_t shiftattn_mixed_workspace_bytes(int32_t num_prefill_seqs, int32_t total_prefill_q, int32_t max_q_len,
                                       int32_t max_prefill_seq_len, int32_t num_decode_seqs, int32_t max_decode_seq_len,
                                       const shiftattn_attn* a) {
    const size_t wp = shiftattn_prefill_workspace_bytes(num_prefill_seqs, total_prefill_q, max_q_len, max_prefill_seq_len, a);
    const size_t wd = shiftattn_decode_workspace_bytes(num_decode_seqs, max_decode_seq_len, a);
    if (wp == SIZE_MAX || wd == SIZE_MAX) return SIZE_MAX;
    return wp > wd ? wp : wd;
}

int shiftattn_mixed(const void* q, const void* k_new, const void* v_new, const int64_t* slot_mapping, void* kv_cache,
                    const int32_t* block_table, const int32_t* cu_seqlens_q, const int32_t* seq_lens,
                    int32_t num_prefill_seqs, int32_t total_prefill_q, int32_t max_q_len, int32_t max_prefill_seq_len,
                    int32_t num_decode_seqs, int32_t max_decode_seq_len, void* out, void* workspace,
                    size_t workspace_bytes, const shiftattn_attn* a, void* stream) {
    AttnShape s;
    if (int rc = check_attn(a, &s)) return rc;
    if (num_prefill_seqs < 0 || total_prefill_q < 0 || max_q_len < 0 || max_prefill_seq_len < 0 || num_decode_seqs < 0 ||
        max_decode_seq_len < 0)
        return fail(SHIFTATTN_EINVAL, "negative size argument");
    if (num_prefill_seqs == 0 && total_prefill_q != 0)
        return fail(SHIFTATTN_EINVAL, "total_prefill_q = %d without prefill sequences", total_prefill_q);
    bool new_kv;
    if (int rc = check_new_kv(k_new, v_new, slot_mapping, &new_kv)) return rc;
    const int64_t rows = static_cast<int64_t>(total_prefill_q) + num_decode_seqs;
    if (rows > INT32_MAX) return fail(SHIFTATTN_EINVAL, "batch of %lld rows is too large", static_cast<long long>(rows));
    if (rows == 0) return SHIFTATTN_OK;
    if (!q || !kv_cache || !block_table || !seq_lens || !out || (num_prefill_seqs > 0 && !cu_seqlens_q))
        return fail(SHIFTATTN_EINVAL, "a required pointer is NULL");
    const size_t need = shiftattn_mixed_workspace_bytes(num_prefill_seqs, total_prefill_q, max_q_len, max_prefill_seq_len,
                                                        num_decode_seqs, max_decode_seq_len, a);
    if (need > 0 && (!workspace || workspace_bytes < need || !aligned16(workspace)))
        return fail(SHIFTATTN_EWORKSPACE, "mixed batch needs %zu workspace bytes, got %zu", need,
                    workspace ? workspace_bytes : static_cast<size_t>(0));
    // everything the two parts would refuse is refused here, before the cache is touched
    const size_t q_off = static_cast<size_t>(total_prefill_q) * s.q_stride * s.elem;
    const size_t o_off = static_cast<size_t>(total_prefill_q) * s.out_stride * s.elem;
    const int32_t* table_d = block_table + static_cast<size_t>(num_prefill_seqs) * s.max_blocks;
    if (int rc = check_prefill_args(q, kv_cache, block_table, cu_seqlens_q, seq_lens, num_prefill_seqs, total_prefill_q,
                                    max_q_len, max_prefill_seq_len, out, s))
        return rc;
    if (int rc = check_decode_args(static_cast<const char*>(q) + q_off, kv_cache, table_d, seq_lens + num_prefill_seqs,
                                   num_decode_seqs, max_decode_seq_len, static_cast<char*>(out) + o_off, s))
        return rc;
    if (new_kv) {
        if (!aligned16(kv_cache)) return fail(SHIFTATTN_EINVAL, "kv_cache must be 16-byte aligned");
        hipError_t e = launch_kv_write(k_new, v_new, slot_mapping, static_cast<int>(rows), kv_cache, s,
                                       static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return hip_fail(e, "kv_write launch");
    }
    // the two kinds of rows go to the kernel built for each; both read the cache written above
    if (int rc = shiftattn_prefill(q, nullptr, nullptr, nullptr, kv_cache, block_table, cu_seqlens_q, seq_lens,
                                   num_prefill_seqs, total_prefill_q, max_q_len, max_prefill_seq_len, out, workspace,
                                   workspace_bytes, a, stream))
        return rc;
    return shiftattn_decode(static_cast<const char*>(q) + q_off, nullptr, nullptr, nullptr, kv_cache, table_d,
                            seq_lens + num_prefill_seqs,
                            num_decode_seqs, max_decode_seq_len, static_cast<char*>(out) + o_off, workspace, workspace_bytes,
                            a, stream);
}

}  // extern "C"
