"""Thin Python binding of the C ABI in include/shiftattn.h.

Argument marshalling only: every function takes torch tensors that already live on the GPU,
checks shapes, and passes raw device pointers plus the current HIP stream to libshiftattn.so.
All of the path's work happens in the library's kernels; there is no Python or CPU fallback.
If the library has not been built (python -m paper_2509_16495_amd.build, or
__graft_entry__.build()), loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SHIFTATTN_LIB") or os.path.join(_HERE, "libshiftattn.so")  # the variable names another build

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP = 0, -1, -2, -3, -4
BF16, F32 = 0, 1
BLOCK_SIZE = 16


class ShiftAttnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"shiftattn error {code}: {msg}")
        self.code = code


class Xchg(ctypes.Structure):
    _fields_ = [("P", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class Attn(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("block_size", ctypes.c_int32), ("num_blocks", ctypes.c_int32),
                ("max_blocks_per_seq", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("q_stride", ctypes.c_int64), ("kv_stride", ctypes.c_int64), ("out_stride", ctypes.c_int64),
                ("kv_format", ctypes.c_int32), ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float),
                ("reserved", ctypes.c_int32)]


KV_SAME, KV_FP8_E4M3 = 0, 1


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """The loaded C library.  Raises if it was never built: there is no other implementation."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2509_16495_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64p, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
        xp, ap = ctypes.POINTER(Xchg), ctypes.POINTER(Attn)
        L.shiftattn_pack_seq2head.argtypes = [vp, vp, i32, i32, xp, vp]
        L.shiftattn_unpack_head2seq.argtypes = [vp, vp, i32, i32, xp, vp]
        L.shiftattn_qkv_proj_pack.argtypes = [vp, vp, vp, i32, i32, i32, xp, vp]
        L.shiftattn_unpack_o_proj.argtypes = [vp, vp, vp, i32, i32, i32, xp, vp]
        L.shiftattn_qkv_proj_pack_ws.argtypes = [vp, vp, vp, i32, i32, i32, xp, vp, ctypes.c_size_t, vp]
        L.shiftattn_unpack_o_proj_ws.argtypes = [vp, vp, vp, i32, i32, i32, xp, vp, ctypes.c_size_t, vp]
        L.shiftattn_proj_workspace_bytes.argtypes = [i32, i32, i32]
        L.shiftattn_proj_workspace_bytes.restype = ctypes.c_size_t
        L.shiftattn_proj_workspace_bytes_fp8.argtypes = [i32, i32, i32]
        L.shiftattn_proj_workspace_bytes_fp8.restype = ctypes.c_size_t
        L.shiftattn_qkv_proj_pack_fp8_ws.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, xp, vp, ctypes.c_size_t, vp]
        L.shiftattn_unpack_o_proj_fp8_ws.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, xp, vp, ctypes.c_size_t, vp]
        L.shiftattn_quantize_rows_fp8.argtypes = [vp, vp, vp, i32, i32, vp]
        L.shiftattn_quantize_recv_fp8.argtypes = [vp, vp, vp, i32, i32, xp, vp]
        L.shiftattn_qkv_proj_pack_fp8.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, xp, vp]
        L.shiftattn_unpack_o_proj_fp8.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, xp, vp]
        L.shiftattn_kv_write.argtypes = [vp, vp, i64p, i32, vp, ap, vp]
        L.shiftattn_prefill.argtypes = [vp, vp, vp, i64p, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, sz, ap, vp]
        L.shiftattn_decode.argtypes = [vp, vp, vp, i64p, vp, vp, vp, i32, i32, vp, vp, sz, ap, vp]
        L.shiftattn_decode_static.argtypes = [vp, vp, vp, i64p, vp, vp, vp, i32, i32, vp, ap, vp]
        L.shiftattn_prefill_workspace_bytes.argtypes = [i32, i32, i32, i32, ap]
        L.shiftattn_prefill_workspace_bytes.restype = sz
        L.shiftattn_decode_workspace_bytes.argtypes = [i32, i32, ap]
        L.shiftattn_decode_workspace_bytes.restype = sz
        L.shiftattn_mixed.argtypes = [vp, vp, vp, i64p, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, sz, ap, vp]
        L.shiftattn_mixed_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32, ap]
        L.shiftattn_mixed_workspace_bytes.restype = sz
        L.shiftattn_head_block.argtypes = [i32, i32, i32]
        L.shiftattn_head_block.restype = i32
        L.shiftattn_kv_head_of_block.argtypes = [i32, i32, i32]
        L.shiftattn_kv_head_of_block.restype = i32
        L.shiftattn_padded_tokens.argtypes = [i32, i32]
        L.shiftattn_padded_tokens.restype = i32
        L.shiftattn_use_base_config.argtypes = [i32, i32]
        L.shiftattn_use_base_config.restype = i32
        L.shiftattn_ceiling_mfma_bf16.argtypes = [vp, vp, i32, ctypes.POINTER(ctypes.c_int64), vp]
        L.shiftattn_ceiling_mfma_bf16_fresh.argtypes = [vp, vp, i32, ctypes.POINTER(ctypes.c_int64), vp]
        L.shiftattn_ceiling_hbm_read.argtypes = [vp, sz, vp, ctypes.POINTER(ctypes.c_int64), vp]
        L.shiftattn_ceiling_hbm_copy.argtypes = [vp, vp, sz, ctypes.POINTER(ctypes.c_int64), vp]
        L.shiftattn_set_option.argtypes = [i32, i32]
        L.shiftattn_get_option.argtypes = [i32]
        L.shiftattn_get_option.restype = i32
        L.shiftattn_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


OPT_PREFILL_TILE, OPT_PREFILL_SPLITS, OPT_GENERIC_ONLY, OPT_PREFILL_PAIRING, OPT_PREFILL_SCALED_Q = 0, 1, 2, 3, 4


def init() -> None:
    _check(lib().shiftattn_init())


def set_option(option: int, value: int) -> None:
    _check(lib().shiftattn_set_option(option, value))


def get_option(option: int) -> int:
    return int(lib().shiftattn_get_option(option))


def last_error() -> str:
    return lib().shiftattn_last_error().decode()


def _check(rc: int) -> None:
    if rc != OK:
        raise ShiftAttnError(rc, last_error())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _row_stride(t: torch.Tensor) -> int:
    """Elements between consecutive tokens of a [tokens, heads, D] view whose inner two dims are dense."""
    assert t.dim() == 3 and t.stride(2) == 1 and (t.shape[1] == 1 or t.stride(1) == t.shape[2]), "inner dims must be dense"
    return int(t.stride(0)) if t.shape[0] > 1 else int(t.shape[1] * t.shape[2])


# ---- host-only helpers --------------------------------------------------------------------------
def head_block(sp: int, tp: int, rank: int) -> int:
    return int(lib().shiftattn_head_block(sp, tp, rank))


def kv_head_of_block(block: int, P: int, h_kv: int) -> int:
    return int(lib().shiftattn_kv_head_of_block(block, P, h_kv))


def padded_tokens(n: int, sp: int) -> int:
    return int(lib().shiftattn_padded_tokens(n, sp))


def use_base_config(n_tokens: int, threshold: int) -> int:
    return int(lib().shiftattn_use_base_config(n_tokens, threshold))


def ceiling_mfma_bf16(operands: torch.Tensor, sink: torch.Tensor, iters: int) -> int:
    """Enqueue the MFMA-only probe; returns the flops of the launch."""
    assert operands.numel() * operands.element_size() >= 2048 and operands.is_contiguous()
    flops = ctypes.c_int64(0)
    _check(lib().shiftattn_ceiling_mfma_bf16(_ptr(operands), _ptr(sink), iters, ctypes.byref(flops), _stream()))
    return flops.value


def ceiling_mfma_bf16_fresh(operands: torch.Tensor, sink: torch.Tensor, iters: int) -> int:
    """Enqueue the MFMA-only probe whose operands change from one MFMA to the next; returns the flops of the launch."""
    assert operands.numel() * operands.element_size() >= 16384 and operands.is_contiguous()
    flops = ctypes.c_int64(0)
    _check(lib().shiftattn_ceiling_mfma_bf16_fresh(_ptr(operands), _ptr(sink), iters, ctypes.byref(flops), _stream()))
    return flops.value


def copy_probe(src: torch.Tensor, dst: torch.Tensor) -> int:
    """Enqueue the read + write streaming probe over all of `src`; returns the bytes copied."""
    assert src.is_contiguous() and dst.is_contiguous() and dst.numel() * dst.element_size() >= src.numel() * src.element_size()
    n = ctypes.c_int64(0)
    _check(lib().shiftattn_ceiling_hbm_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), ctypes.byref(n), _stream()))
    return n.value


def ceiling_hbm_read(src: torch.Tensor, sink: torch.Tensor) -> int:
    """Enqueue the streaming-read probe over all of `src`; returns the bytes requested."""
    assert src.is_contiguous()
    n = ctypes.c_int64(0)
    _check(lib().shiftattn_ceiling_hbm_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), ctypes.byref(n),
                                            _stream()))
    return n.value


def local_kv_heads(P: int, h_kv: int) -> int:
    return 0 if h_kv == 0 else (h_kv // P if h_kv >= P else 1)


# ---- exchange pack / unpack -----------------------------------------------------------------------
def pack_seq2head(qkv: torch.Tensor, send: torch.Tensor, P: int, h: int, h_kv: int) -> None:
    """qkv [T, h+2*h_kv, D] -> send [P, T_pad, h/P + 2*hkv_l, D] (pad rows zeroed)."""
    T, w, D = qkv.shape
    assert w == h + 2 * h_kv and qkv.is_contiguous() and send.is_contiguous() and send.dtype == qkv.dtype
    T_pad = send.shape[1]
    assert send.shape[0] == P and send.shape[3] == D
    x = Xchg(P, h, h_kv, D, _dtype_code(qkv))
    _check(lib().shiftattn_pack_seq2head(_ptr(qkv), _ptr(send), T, T_pad, ctypes.byref(x), _stream()))


def unpack_head2seq(recv: torch.Tensor, out: torch.Tensor) -> None:
    """recv [P, T_pad, h/P, D] -> out [T, h, D]."""
    P, T_pad, hq_l, D = recv.shape
    T, h, D2 = out.shape
    assert D2 == D and h == P * hq_l and recv.is_contiguous() and out.is_contiguous() and out.dtype == recv.dtype
    x = Xchg(P, h, 0, D, _dtype_code(recv))
    _check(lib().shiftattn_unpack_head2seq(_ptr(recv), _ptr(out), T, T_pad, ctypes.byref(x), _stream()))


# ---- KV cache and attention -------------------------------------------------------------------------
def proj_workspace_bytes(rows: int, n_features: int, k: int, fp8: bool = False) -> int:
    """Bytes of workspace that make a projection of `rows` token rows with an [n_features, k] matrix one pass over the weights."""
    if fp8:
        return int(lib().shiftattn_proj_workspace_bytes_fp8(rows, n_features, k))
    return int(lib().shiftattn_proj_workspace_bytes(rows, n_features, k))


def qkv_proj_pack(x: torch.Tensor, w_qkv: torch.Tensor, send: torch.Tensor, P: int, h: int, h_kv: int,
                  workspace: Optional[torch.Tensor] = None) -> None:
    """x [T, d_model], w_qkv [(h + 2 h_kv) D, d_model] -> send [P, T_pad, hq_l + 2 hkv_l, D] (projection + pack)."""
    T, d_model = x.shape
    T_pad, D = send.shape[1], send.shape[3]
    assert w_qkv.shape == ((h + 2 * h_kv) * D, d_model) and x.is_contiguous() and w_qkv.is_contiguous() and send.is_contiguous()
    assert send.shape[0] == P and send.shape[2] == h // P + 2 * local_kv_heads(P, h_kv) and x.dtype == w_qkv.dtype == send.dtype
    xc = Xchg(P, h, h_kv, D, _dtype_code(x))
    if workspace is None:
        _check(lib().shiftattn_qkv_proj_pack(_ptr(x), _ptr(w_qkv), _ptr(send), T, T_pad, d_model, ctypes.byref(xc), _stream()))
    else:
        _check(lib().shiftattn_qkv_proj_pack_ws(_ptr(x), _ptr(w_qkv), _ptr(send), T, T_pad, d_model, ctypes.byref(xc), _ptr(workspace),
                                                workspace.numel() * workspace.element_size(), _stream()))


def unpack_o_proj(recv: torch.Tensor, w_o: torch.Tensor, out: torch.Tensor, workspace: Optional[torch.Tensor] = None) -> None:
    """recv [P, T_pad, hq_l, D], w_o [d_model, h D] -> out [T, d_model] (unpack + projection)."""
    P, T_pad, hq_l, D = recv.shape
    T, d_model = out.shape
    assert w_o.shape == (d_model, P * hq_l * D) and recv.is_contiguous() and w_o.is_contiguous() and out.is_contiguous()
    assert recv.dtype == w_o.dtype == out.dtype
    xc = Xchg(P, P * hq_l, 0, D, _dtype_code(recv))
    if workspace is None:
        _check(lib().shiftattn_unpack_o_proj(_ptr(recv), _ptr(w_o), _ptr(out), T, T_pad, d_model, ctypes.byref(xc), _stream()))
    else:
        _check(lib().shiftattn_unpack_o_proj_ws(_ptr(recv), _ptr(w_o), _ptr(out), T, T_pad, d_model, ctypes.byref(xc), _ptr(workspace),
                                                workspace.numel() * workspace.element_size(), _stream()))


def quantize_rows_fp8(x: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor) -> None:
    """x [rows, cols] bf16 -> codes [rows, cols] uint8 (FP8 E4M3), scales [rows] float32 (amax / 448)."""
    rows, cols = x.shape
    assert x.dtype == torch.bfloat16 and codes.dtype == torch.uint8 and scales.dtype == torch.float32
    assert codes.shape == x.shape and scales.shape == (rows,) and x.is_contiguous() and codes.is_contiguous() and scales.is_contiguous()
    _check(lib().shiftattn_quantize_rows_fp8(_ptr(x), _ptr(codes), _ptr(scales), rows, cols, _stream()))


def quantize_recv_fp8(recv: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor) -> None:
    """recv [P, T_pad, hq_l, D] bf16 -> codes of the same shape (uint8), scales [T]: one scale per token over all buffers."""
    P, T_pad, hq_l, D = recv.shape
    T = scales.shape[0]
    assert recv.dtype == torch.bfloat16 and codes.dtype == torch.uint8 and scales.dtype == torch.float32 and codes.shape == recv.shape
    assert recv.is_contiguous() and codes.is_contiguous() and scales.is_contiguous()
    xc = Xchg(P, P * hq_l, 0, D, BF16)
    _check(lib().shiftattn_quantize_recv_fp8(_ptr(recv), _ptr(codes), _ptr(scales), T, T_pad, ctypes.byref(xc), _stream()))


def qkv_proj_pack_fp8(x_codes: torch.Tensor, x_scales: torch.Tensor, w_codes: torch.Tensor, w_scales: torch.Tensor,
                      send: torch.Tensor, P: int, h: int, h_kv: int, workspace: Optional[torch.Tensor] = None) -> None:
    """FP8 E4M3 codes x [T, d_model] and w [(h + 2 h_kv) D, d_model] with their row scales -> bf16 send buffers."""
    T, d_model = x_codes.shape
    T_pad, D = send.shape[1], send.shape[3]
    assert x_codes.dtype == w_codes.dtype == torch.uint8 and x_scales.dtype == w_scales.dtype == torch.float32 and send.dtype == torch.bfloat16
    assert w_codes.shape == ((h + 2 * h_kv) * D, d_model) and x_scales.shape == (T,) and w_scales.shape == (w_codes.shape[0],)
    assert send.shape[0] == P and send.shape[2] == h // P + 2 * local_kv_heads(P, h_kv)
    assert all(t.is_contiguous() for t in (x_codes, x_scales, w_codes, w_scales, send))
    xc = Xchg(P, h, h_kv, D, BF16)
    _check(lib().shiftattn_qkv_proj_pack_fp8_ws(_ptr(x_codes), _ptr(x_scales), _ptr(w_codes), _ptr(w_scales), _ptr(send), T, T_pad,
                                                d_model, ctypes.byref(xc), _ptr(workspace) if workspace is not None else None,
                                                workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()))


def unpack_o_proj_fp8(recv_codes: torch.Tensor, a_scales: torch.Tensor, w_codes: torch.Tensor, w_scales: torch.Tensor,
                      out: torch.Tensor, workspace: Optional[torch.Tensor] = None) -> None:
    """FP8 E4M3 codes recv [P, T_pad, hq_l, D] (one scale per token) and w [d_model, h D] (one per feature) -> out [T, d_model] bf16."""
    P, T_pad, hq_l, D = recv_codes.shape
    T, d_model = out.shape
    assert recv_codes.dtype == w_codes.dtype == torch.uint8 and a_scales.dtype == w_scales.dtype == torch.float32 and out.dtype == torch.bfloat16
    assert w_codes.shape == (d_model, P * hq_l * D) and a_scales.shape[0] >= T and w_scales.shape == (d_model,)
    assert all(t.is_contiguous() for t in (recv_codes, a_scales, w_codes, w_scales, out))
    xc = Xchg(P, P * hq_l, 0, D, BF16)
    _check(lib().shiftattn_unpack_o_proj_fp8_ws(_ptr(recv_codes), _ptr(a_scales), _ptr(w_codes), _ptr(w_scales), _ptr(out), T, T_pad,
                                                d_model, ctypes.byref(xc), _ptr(workspace) if workspace is not None else None,
                                                workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream()))


def attn_desc(q: torch.Tensor, kv_cache: torch.Tensor, block_table: torch.Tensor, softmax_scale: float,
              k_new: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None, k_scale: float = 1.0,
              v_scale: float = 1.0) -> Attn:
    """Descriptor from tensor shapes.  kv_cache is [num_blocks, hkv_l, 2, 16*D] in q's type, or uint8 for an
    FP8 E4M3 cache (then k_scale / v_scale give the value of a code)."""
    hq_l, D = q.shape[1], q.shape[2]
    num_blocks, hkv_l, two, bd = kv_cache.shape
    fp8 = kv_cache.dtype == torch.uint8
    assert two == 2 and bd == BLOCK_SIZE * D and kv_cache.is_contiguous() and (fp8 or kv_cache.dtype == q.dtype)
    assert block_table.dtype == torch.int32 and block_table.dim() == 2 and block_table.is_contiguous()
    a = Attn(hq_l, hkv_l, D, _dtype_code(q), BLOCK_SIZE, num_blocks, block_table.shape[1], float(softmax_scale),
             _row_stride(q), 0, 0, KV_FP8_E4M3 if fp8 else KV_SAME, float(k_scale), float(v_scale), 0)
    if k_new is not None:
        a.kv_stride = _row_stride(k_new)
    if out is not None:
        a.out_stride = _row_stride(out)
    return a


def kv_write(k_new: torch.Tensor, v_new: torch.Tensor, slot_mapping: torch.Tensor, kv_cache: torch.Tensor,
             k_scale: float = 1.0, v_scale: float = 1.0) -> None:
    n, hkv_l, D = k_new.shape
    assert v_new.shape == k_new.shape and slot_mapping.dtype == torch.int64 and slot_mapping.shape[0] == n
    assert _row_stride(v_new) == _row_stride(k_new)
    num_blocks = kv_cache.shape[0]
    assert kv_cache.shape[1:] == (hkv_l, 2, BLOCK_SIZE * D) and kv_cache.is_contiguous()
    fp8 = kv_cache.dtype == torch.uint8
    a = Attn(hkv_l, hkv_l, D, _dtype_code(k_new), BLOCK_SIZE, num_blocks, 0, 1.0, 0, _row_stride(k_new), 0,
             KV_FP8_E4M3 if fp8 else KV_SAME, float(k_scale), float(v_scale), 0)
    _check(lib().shiftattn_kv_write(_ptr(k_new), _ptr(v_new), _ptr(slot_mapping), n, _ptr(kv_cache), ctypes.byref(a),
                                    _stream()))


def prefill_workspace_bytes(num_seqs: int, total_q: int, max_q_len: int, max_seq_len: int, a: Attn) -> int:
    return int(lib().shiftattn_prefill_workspace_bytes(num_seqs, total_q, max_q_len, max_seq_len, ctypes.byref(a)))


def decode_workspace_bytes(num_seqs: int, max_seq_len: int, a: Attn) -> int:
    return int(lib().shiftattn_decode_workspace_bytes(num_seqs, max_seq_len, ctypes.byref(a)))


def prefill(q: torch.Tensor, kv_cache: torch.Tensor, block_table: torch.Tensor, cu_seqlens_q: torch.Tensor,
            seq_lens: torch.Tensor, max_q_len: int, max_seq_len: int, out: torch.Tensor, softmax_scale: float,
            k_new: Optional[torch.Tensor] = None, v_new: Optional[torch.Tensor] = None,
            slot_mapping: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, k_scale: float = 1.0,
            v_scale: float = 1.0) -> None:
    """Causal attention of prefill chunks; q/out [total_q, hq_l, D] (row-strided views allowed)."""
    total_q = q.shape[0]
    num_seqs = seq_lens.shape[0]
    assert cu_seqlens_q.dtype == torch.int32 and seq_lens.dtype == torch.int32 and cu_seqlens_q.shape[0] == num_seqs + 1
    assert out.shape == q.shape and out.dtype == q.dtype
    a = attn_desc(q, kv_cache, block_table, softmax_scale, k_new, out, k_scale, v_scale)
    need = prefill_workspace_bytes(num_seqs, total_q, max_q_len, max_seq_len, a)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().shiftattn_prefill(_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(slot_mapping), _ptr(kv_cache),
                                   _ptr(block_table), _ptr(cu_seqlens_q), _ptr(seq_lens), num_seqs, total_q,
                                   max_q_len, max_seq_len, _ptr(out), _ptr(workspace), ws_bytes, ctypes.byref(a),
                                   _stream()))


def decode(q: torch.Tensor, kv_cache: torch.Tensor, block_table: torch.Tensor, seq_lens: torch.Tensor,
           max_seq_len: int, out: torch.Tensor, softmax_scale: float, k_new: Optional[torch.Tensor] = None,
           v_new: Optional[torch.Tensor] = None, slot_mapping: Optional[torch.Tensor] = None,
           workspace: Optional[torch.Tensor] = None, k_scale: float = 1.0, v_scale: float = 1.0) -> None:
    """One new token per sequence; q/out [num_seqs, hq_l, D]."""
    num_seqs = q.shape[0]
    assert seq_lens.dtype == torch.int32 and seq_lens.shape[0] == num_seqs
    assert out.shape == q.shape and out.dtype == q.dtype
    a = attn_desc(q, kv_cache, block_table, softmax_scale, k_new, out, k_scale, v_scale)
    need = decode_workspace_bytes(num_seqs, max_seq_len, a)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().shiftattn_decode(_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(slot_mapping), _ptr(kv_cache),
                                  _ptr(block_table), _ptr(seq_lens), num_seqs, max_seq_len, _ptr(out),
                                  _ptr(workspace), ws_bytes, ctypes.byref(a), _stream()))


STATIC_SCRATCH_BYTES = 16 << 20


def decode_static(q: torch.Tensor, kv_cache: torch.Tensor, block_table: torch.Tensor, seq_lens: torch.Tensor,
                  max_seq_len: int, out: torch.Tensor, softmax_scale: float, k_new: Optional[torch.Tensor] = None,
                  v_new: Optional[torch.Tensor] = None, slot_mapping: Optional[torch.Tensor] = None, k_scale: float = 1.0,
                  v_scale: float = 1.0) -> None:
    """decode() without a workspace: the library's own static device array takes the split partials."""
    num_seqs = q.shape[0]
    assert seq_lens.dtype == torch.int32 and seq_lens.shape[0] == num_seqs
    assert out.shape == q.shape and out.dtype == q.dtype
    a = attn_desc(q, kv_cache, block_table, softmax_scale, k_new, out, k_scale, v_scale)
    _check(lib().shiftattn_decode_static(_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(slot_mapping), _ptr(kv_cache),
                                         _ptr(block_table), _ptr(seq_lens), num_seqs, max_seq_len, _ptr(out),
                                         ctypes.byref(a), _stream()))


def mixed_workspace_bytes(num_prefill_seqs: int, total_prefill_q: int, max_q_len: int, max_prefill_seq_len: int,
                          num_decode_seqs: int, max_decode_seq_len: int, a: Attn) -> int:
    return int(lib().shiftattn_mixed_workspace_bytes(num_prefill_seqs, total_prefill_q, max_q_len, max_prefill_seq_len,
                                                     num_decode_seqs, max_decode_seq_len, ctypes.byref(a)))


def mixed(q: torch.Tensor, kv_cache: torch.Tensor, block_table: torch.Tensor, cu_seqlens_q: torch.Tensor,
          seq_lens: torch.Tensor, num_prefill_seqs: int, max_q_len: int, max_prefill_seq_len: int,
          max_decode_seq_len: int, out: torch.Tensor, softmax_scale: float, k_new: Optional[torch.Tensor] = None,
          v_new: Optional[torch.Tensor] = None, slot_mapping: Optional[torch.Tensor] = None,
          workspace: Optional[torch.Tensor] = None, k_scale: float = 1.0, v_scale: float = 1.0) -> None:
    """Unified batch: the first num_prefill_seqs sequences are chunks (cu_seqlens_q [num_prefill_seqs + 1]), the
    others carry one row each; q/out hold the chunk rows first, then the decode rows."""
    num_decode_seqs = seq_lens.shape[0] - num_prefill_seqs
    total_prefill_q = q.shape[0] - num_decode_seqs
    assert num_decode_seqs >= 0 and total_prefill_q >= 0 and cu_seqlens_q.shape[0] == num_prefill_seqs + 1
    assert cu_seqlens_q.dtype == torch.int32 and seq_lens.dtype == torch.int32
    assert out.shape == q.shape and out.dtype == q.dtype and block_table.shape[0] == seq_lens.shape[0]
    a = attn_desc(q, kv_cache, block_table, softmax_scale, k_new, out, k_scale, v_scale)
    need = mixed_workspace_bytes(num_prefill_seqs, total_prefill_q, max_q_len, max_prefill_seq_len, num_decode_seqs,
                                 max_decode_seq_len, a)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().shiftattn_mixed(_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(slot_mapping), _ptr(kv_cache), _ptr(block_table),
                                 _ptr(cu_seqlens_q), _ptr(seq_lens), num_prefill_seqs, total_prefill_q, max_q_len,
                                 max_prefill_seq_len, num_decode_seqs, max_decode_seq_len, _ptr(out), _ptr(workspace),
                                 ws_bytes, ctypes.byref(a), _stream()))


# ---- numpy <-> device helpers for tests and benchmarks (storage only) ------------------------------------
def to_device(a, dtype: str, device: str = "cuda:0") -> torch.Tensor:
    """numpy array in the workloads storage convention (uint16 bit patterns for bf16) -> GPU tensor."""
    import numpy as np
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def to_host(t: torch.Tensor):
    """GPU tensor -> numpy array in the workloads storage convention."""
    import numpy as np
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
