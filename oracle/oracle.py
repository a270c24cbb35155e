"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.
It loads `liboracle.so` (built from `shiftattn_oracle.c` with gcc) through
ctypes and adds a few steps that are plain numpy: the virtual-rank exchange,
the split-K merge identity, and a second, independent numpy statement of
attention for tiny inputs.  Nothing here imports or calls the HIP path.

Citations are to the paper: Algorithm 1 (combined SP,TP forward), Sec. 2.2
(attention and KV cache), Sec. 3.2.1 (GQA, KV replication, padding),
Sec. 3.3.1 / 3.3.2 (head order, process groups).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "shiftattn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

DTYPE_CODE = {"bf16": 0, "f32": 1, "fp8_e4m3": 2}
_NP_STORE = {"bf16": np.uint16, "f32": np.float32, "fp8_e4m3": np.uint8}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no -march flags: the library travels between hosts)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        L = ctypes.CDLL(_LIB)
        i32, i64, vp, dbl = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_double
        L.oracle_num_threads.restype = i32
        L.oracle_head_block.argtypes = [i32, i32, i32]
        L.oracle_kv_head_of_block.argtypes = [i32, i32, i32]
        L.oracle_pack_seq2head.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32]
        L.oracle_unpack_head2seq.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32]
        L.oracle_kv_write.argtypes = [vp, vp, vp, i64, vp, i32, i32, i32, i32]
        L.oracle_attention.argtypes = [vp, vp, i32, vp, i32, vp, vp, i32, i32, i32, i32, i32, dbl, vp, i64, vp]
        flt, u8 = ctypes.c_float, ctypes.c_uint8
        L.oracle_kv_write_fp8.argtypes = [vp, vp, vp, i64, vp, i32, i32, i32, i32, flt, flt]
        L.oracle_attention_kv.argtypes = [vp, i32, vp, i32, dbl, dbl, vp, i32, vp, vp, i32, i32, i32, i32, i32, dbl, vp,
                                          i64, vp]
        L.oracle_quantize_rows_e4m3.argtypes = [vp, i32, i64, i64, i64, vp, vp]
        L.oracle_e4m3_value.argtypes = [u8]
        L.oracle_e4m3_value.restype = dbl
        L.oracle_e4m3_from_float.argtypes = [flt]
        L.oracle_e4m3_from_float.restype = u8
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


# ---------------------------------------------------------------------------
# head / rank maps (Sec. 3.3.1, 3.3.2)
# ---------------------------------------------------------------------------
def head_block(sp: int, tp: int, rank: int) -> int:
    return int(lib().oracle_head_block(sp, tp, rank))


def kv_head_of_block(p: int, P: int, h_kv: int) -> int:
    return int(lib().oracle_kv_head_of_block(p, P, h_kv))


def process_groups(sp: int, tp: int):
    """TP groups: consecutive ranks; SP groups: every TP-th rank; SP_TP: the SP groups one
    after another, i.e. ranks listed in the order of the head block they hold."""
    tp_groups = [[s * tp + t for t in range(tp)] for s in range(sp)]
    sp_groups = [[s * tp + t for s in range(sp)] for t in range(tp)]
    sp_tp = [[r for g in sp_groups for r in g]]
    return tp_groups, sp_groups, sp_tp


def local_kv_heads(P: int, h_kv: int) -> int:
    return 0 if h_kv == 0 else (h_kv // P if h_kv >= P else 1)


# ---------------------------------------------------------------------------
# pack / exchange / unpack (Algorithm 1, the two SP all-to-all lines)
# ---------------------------------------------------------------------------
def pack_seq2head(x: np.ndarray, P: int, h: int, h_kv: int, T_pad: int, dtype: str) -> np.ndarray:
    T, w_in, D = x.shape
    assert w_in == h + 2 * h_kv
    hq_l, hkv_l = h // P, local_kv_heads(P, h_kv)
    x = np.ascontiguousarray(x, dtype=_NP_STORE[dtype])
    send = np.empty((P, T_pad, hq_l + 2 * hkv_l, D), dtype=_NP_STORE[dtype])
    send.view(np.uint8)[...] = 0x55  # poison: the pack must define every byte, pad rows included
    rc = lib().oracle_pack_seq2head(_p(x), _p(send), T, T_pad, P, h, h_kv, D, DTYPE_CODE[dtype])
    assert rc == 0
    return send


def exchange(send_of_rank: Sequence[np.ndarray], r: int) -> np.ndarray:
    """What member r of the exchange group holds after the all-to-all: the r-th send buffer of
    every member, concatenated in member order (rows of member 0 first).  Pure data movement."""
    return np.concatenate([s[r] for s in send_of_rank], axis=0)


def unpack_head2seq(recv: np.ndarray, T: int, dtype: str) -> np.ndarray:
    P, T_pad, hq_l, D = recv.shape
    recv = np.ascontiguousarray(recv, dtype=_NP_STORE[dtype])
    out = np.empty((T, P * hq_l, D), dtype=_NP_STORE[dtype])
    out.view(np.uint8)[...] = 0x55
    rc = lib().oracle_unpack_head2seq(_p(recv), _p(out), T, T_pad, P, P * hq_l, D, DTYPE_CODE[dtype])
    assert rc == 0
    return out


# ---------------------------------------------------------------------------
# the projections next to the exchange (Algorithm 1: qkv = embed * W_qkv before the first all-to-all,
# embed = attn_o * W_o after the second).  float64 over the stored values; the layouts are the pack /
# unpack above restated on float64 arrays.
# ---------------------------------------------------------------------------
def _stored_to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of stored values (bf16 as uint16 bit patterns, or float32) to float64."""
    if dtype == "bf16":
        return (np.ascontiguousarray(a, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def pack_heads_f64(y: np.ndarray, P: int, h: int, h_kv: int, T_pad: int) -> np.ndarray:
    """y [T, h + 2 h_kv, D] float64 -> send [P, T_pad, hq_l + 2 hkv_l, D]; pad rows zero."""
    T, w_in, D = y.shape
    assert w_in == h + 2 * h_kv and h % P == 0
    hq_l, hkv_l = h // P, local_kv_heads(P, h_kv)
    send = np.zeros((P, T_pad, hq_l + 2 * hkv_l, D), dtype=np.float64)
    for p in range(P):
        send[p, :T, :hq_l] = y[:, p * hq_l:(p + 1) * hq_l]
        if h_kv:
            kv0 = kv_head_of_block(p, P, h_kv)
            send[p, :T, hq_l:hq_l + hkv_l] = y[:, h + kv0:h + kv0 + hkv_l]
            send[p, :T, hq_l + hkv_l:] = y[:, h + h_kv + kv0:h + h_kv + kv0 + hkv_l]
    return send


def qkv_proj_pack(x: np.ndarray, w_qkv: np.ndarray, P: int, h: int, h_kv: int, D: int, T_pad: int, dtype: str) -> np.ndarray:
    """x [T, d] and w_qkv [(h + 2 h_kv) D, d] (one row per output feature, as weights are stored) in `dtype`;
    returns the float64 send buffers of the first all-to-all."""
    x64, w64 = _stored_to_f64(x, dtype), _stored_to_f64(w_qkv, dtype)
    y = x64 @ w64.T
    return pack_heads_f64(y.reshape(x.shape[0], h + 2 * h_kv, D), P, h, h_kv, T_pad)


def unpack_o_proj(recv: np.ndarray, w_o: np.ndarray, T: int, dtype: str) -> np.ndarray:
    """recv [P, T_pad, hq_l, D] (what the second all-to-all delivers) and w_o [d, h D] in `dtype`;
    returns embed [T, d] float64 = unpack(recv) * W_o^T."""
    P, T_pad, hq_l, D = recv.shape
    r64 = _stored_to_f64(recv, dtype)
    a = np.concatenate([r64[p, :T] for p in range(P)], axis=1).reshape(T, P * hq_l * D)  # out[t, p hq_l + j] = recv[p][t][j]
    return a @ _stored_to_f64(w_o, dtype).T


# ---- the same projections with FP8 E4M3 operands (Sec. 4.1 serves FP8 models; scale rule: this build's reading) ----
def quantize_rows_e4m3(x: np.ndarray, dtype: str):
    """x [rows, cols] stored in `dtype` -> (codes uint8 [rows, cols], scales float32 [rows]): scale = amax / 448 in
    float32 (1 for a zero row), code = E4M3 code nearest to the float32 quotient x / scale."""
    x = np.ascontiguousarray(x, dtype=_NP_STORE[dtype])
    rows, cols = x.shape
    codes = np.empty((rows, cols), dtype=np.uint8)
    scales = np.empty(rows, dtype=np.float32)
    rc = lib().oracle_quantize_rows_e4m3(_p(x), DTYPE_CODE[dtype], rows, cols, cols, _p(codes), _p(scales))
    assert rc == 0
    return codes, scales


def e4m3_table() -> np.ndarray:
    return np.array([e4m3_value(c) for c in range(256)], dtype=np.float64)


def recv_rows(recv: np.ndarray, T: int) -> np.ndarray:
    """recv [P, T_pad, hq_l, D] -> [T, P hq_l D]: token t's attention output, heads in global order."""
    P, T_pad, hq_l, D = recv.shape
    return np.concatenate([recv[p, :T].reshape(T, hq_l * D) for p in range(P)], axis=1)


def qkv_proj_pack_fp8(x_codes, x_scales, w_codes, w_scales, P: int, h: int, h_kv: int, D: int, T_pad: int) -> np.ndarray:
    """y[t][f] = x_scale[t] w_scale[f] sum_k value(x_codes[t][k]) value(w_codes[f][k]) in float64, packed like qkv_proj_pack."""
    tab = e4m3_table()
    y = (tab[x_codes] @ tab[w_codes].T) * x_scales.astype(np.float64)[:, None] * w_scales.astype(np.float64)[None, :]
    return pack_heads_f64(y.reshape(x_codes.shape[0], h + 2 * h_kv, D), P, h, h_kv, T_pad)


def unpack_o_proj_fp8(recv_codes, a_scales, w_codes, w_scales, T: int) -> np.ndarray:
    """recv_codes [P, T_pad, hq_l, D] uint8 with one scale per token; w_codes [d, h D] with one scale per output feature."""
    tab = e4m3_table()
    a = tab[recv_rows(recv_codes, T)]
    return (a @ tab[w_codes].T) * a_scales.astype(np.float64)[:T, None] * w_scales.astype(np.float64)[None, :]


# ---------------------------------------------------------------------------
# KV cache
# ---------------------------------------------------------------------------
def new_cache(num_blocks: int, hkv_l: int, B: int, D: int, dtype: str, fill_byte: int = 0xA5) -> np.ndarray:
    """Cache array [num_blocks, hkv_l, 2, B*D] filled with a sentinel byte pattern."""
    c = np.empty((num_blocks, hkv_l, 2, B * D), dtype=_NP_STORE[dtype])
    c.view(np.uint8)[...] = fill_byte
    return c


def kv_write(cache: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, slots: np.ndarray, B: int, dtype: str) -> None:
    n, hkv_l, D = k_new.shape
    k_new = np.ascontiguousarray(k_new, dtype=_NP_STORE[dtype])
    v_new = np.ascontiguousarray(v_new, dtype=_NP_STORE[dtype])
    slots = np.ascontiguousarray(slots, dtype=np.int64)
    assert cache.flags.c_contiguous and cache.shape[1] == hkv_l and cache.shape[3] == B * D
    rc = lib().oracle_kv_write(_p(k_new), _p(v_new), _p(slots), n, _p(cache), hkv_l, D, B, DTYPE_CODE[dtype])
    assert rc == 0


def e4m3_value(code: int) -> float:
    return float(lib().oracle_e4m3_value(int(code) & 0xFF))


def e4m3_from_float(x: float) -> int:
    return int(lib().oracle_e4m3_from_float(float(np.float32(x))))


def kv_write_fp8(cache: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, slots: np.ndarray, B: int, src_dtype: str,
                 k_scale: float, v_scale: float) -> None:
    """Append into an FP8 E4M3 cache (uint8 [num_blocks, hkv_l, 2, B*D]); k_new/v_new stored in src_dtype."""
    n, hkv_l, D = k_new.shape
    k_new = np.ascontiguousarray(k_new, dtype=_NP_STORE[src_dtype])
    v_new = np.ascontiguousarray(v_new, dtype=_NP_STORE[src_dtype])
    slots = np.ascontiguousarray(slots, dtype=np.int64)
    assert cache.dtype == np.uint8 and cache.flags.c_contiguous and cache.shape[1] == hkv_l and cache.shape[3] == B * D
    rc = lib().oracle_kv_write_fp8(_p(k_new), _p(v_new), _p(slots), n, _p(cache), hkv_l, D, B, DTYPE_CODE[src_dtype],
                                   float(k_scale), float(v_scale))
    assert rc == 0


# ---------------------------------------------------------------------------
# attention (Algorithm 1 boxed line; Sec. 2.2)
# ---------------------------------------------------------------------------
def attention(q: np.ndarray, cache: np.ndarray, dtype: str, block_table: np.ndarray, cu_seqlens_q: np.ndarray,
              seq_lens: np.ndarray, hq_l: int, hkv_l: int, D: int, B: int, scale: float,
              rows: Optional[np.ndarray] = None, kv_dtype: Optional[str] = None, k_scale: float = 1.0,
              v_scale: float = 1.0) -> np.ndarray:
    """kv_dtype: how the cache is stored when it differs from q's type ("fp8_e4m3" with its two scales)."""
    kv_dtype = kv_dtype or dtype
    assert cache.dtype == _NP_STORE[kv_dtype]
    q = np.ascontiguousarray(q, dtype=_NP_STORE[dtype])
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    cu = np.ascontiguousarray(cu_seqlens_q, dtype=np.int32)
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    S = sl.shape[0]
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        n_rows = rows.shape[0]
    else:
        n_rows = int(cu[-1]) if S else 0
    out = np.zeros((n_rows, hq_l, D), dtype=np.float64)
    if n_rows == 0:
        return out
    rc = lib().oracle_attention_kv(_p(q), DTYPE_CODE[dtype], _p(cache), DTYPE_CODE[kv_dtype], float(k_scale),
                                   float(v_scale), _p(block_table), block_table.shape[1], _p(cu), _p(sl), S, hq_l, hkv_l,
                                   D, B, float(scale), _p(rows), n_rows, _p(out))
    assert rc == 0, "oracle_attention: inconsistent arguments"
    return out


def attention_case(case, cache: np.ndarray, rows: Optional[np.ndarray] = None, k_scale: float = 1.0,
                   v_scale: float = 1.0) -> np.ndarray:
    """Attention for a workloads.AttnCase over an already written cache (a uint8 cache is read as FP8 E4M3)."""
    kv_dtype = "fp8_e4m3" if cache.dtype == np.uint8 else case.dtype
    return attention(case.q, cache, case.dtype, case.block_table, case.cu_seqlens_q, case.ctx_lens,
                     case.hq_l, case.hkv_l, case.D, case.block_size, case.softmax_scale, rows, kv_dtype, k_scale, v_scale)


def cache_for_case(case, only_cached: bool = False, fp8_scales: Optional[Sequence[float]] = None) -> np.ndarray:
    """Sentinel-filled cache with the case's context written through kv_write.
    only_cached=True leaves out the new tokens (their K/V arrive with the call under test).
    fp8_scales=(k_scale, v_scale): an FP8 E4M3 cache instead of one in the case's own type."""
    slots = case.slots
    if only_cached:
        slots = slots.copy()
        slots[case.new_token_index] = -1
    if fp8_scales is not None:
        cache = new_cache(case.num_blocks, case.hkv_l, case.block_size, case.D, "fp8_e4m3")
        kv_write_fp8(cache, case.k_ctx, case.v_ctx, slots, case.block_size, case.dtype, fp8_scales[0], fp8_scales[1])
        return cache
    cache = new_cache(case.num_blocks, case.hkv_l, case.block_size, case.D, case.dtype)
    kv_write(cache, case.k_ctx, case.v_ctx, slots, case.block_size, case.dtype)
    return cache


# ---------------------------------------------------------------------------
# numpy statements used to pin the C code on tiny inputs
# ---------------------------------------------------------------------------
def attention_dense_np(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float, q_len: int) -> np.ndarray:
    """One sequence, dense float64 K,V [ctx, hkv, D], q [q_len, hq, D]; bottom-right causal mask.
    softmax(scale * Q K^T + mask) V written with numpy primitives."""
    ctx, hkv, D = k.shape
    hq = q.shape[1]
    group = hq // hkv
    out = np.zeros((q_len, hq, D))
    for j in range(hq):
        g = j // group
        s = scale * (q[:, j, :] @ k[:, g, :].T)                 # [q_len, ctx]
        pos = ctx - q_len + np.arange(q_len)[:, None]
        s = np.where(np.arange(ctx)[None, :] <= pos, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=1, keepdims=True)
        out[:, j, :] = p @ v[:, g, :]
    return out


def splitk_partials(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float, bounds: Sequence[int]):
    """Per key-range partial results (m, l, o) of one query vector q[D] against k,v[ctx, D]:
    m = max logit, l = sum exp(logit - m), o = sum exp(logit - m) * v over the range."""
    parts = []
    for a, b in zip(bounds[:-1], bounds[1:]):
        s = scale * (k[a:b] @ q)
        m = s.max()
        e = np.exp(s - m)
        parts.append((m, e.sum(), e @ v[a:b]))
    return parts


def splitk_combine(parts) -> np.ndarray:
    """Merge partials in list order: m* = max m_c, l* = sum l_c e^{m_c-m*}, o = sum o_c e^{m_c-m*} / l*."""
    m_star = max(p[0] for p in parts)
    l_star = 0.0
    o = np.zeros_like(parts[0][2])
    for m, l, oc in parts:
        w = np.exp(m - m_star)
        l_star += l * w
        o = o + oc * w
    return o / l_star
