"""Drives the HIP path through its Python binding with numpy in / numpy out, mirroring the call
shapes of the CPU oracle so that one scenario can be run on both.  Used by GPU tests only."""
from __future__ import annotations

import numpy as np
import torch

from paper_2509_16495_amd import binding as B

DEV = "cuda:0"


def t(a: np.ndarray, dtype: str) -> torch.Tensor:
    return B.to_device(a, dtype, DEV)


def ti(a: np.ndarray, np_dtype) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np_dtype)).to(DEV)


def torch_dtype(dtype: str):
    return {"bf16": torch.bfloat16, "f32": torch.float32}[dtype]


def pack_seq2head(x: np.ndarray, P: int, h: int, h_kv: int, T_pad: int, dtype: str) -> np.ndarray:
    T, w, D = x.shape
    hq_l, hkv_l = h // P, B.local_kv_heads(P, h_kv)
    send = torch.empty((P, T_pad, hq_l + 2 * hkv_l, D), dtype=torch_dtype(dtype), device=DEV)
    send.view(torch.uint8).fill_(0x55)
    B.pack_seq2head(t(x, dtype), send, P, h, h_kv)
    torch.cuda.synchronize()
    return B.to_host(send)


def unpack_head2seq(recv: np.ndarray, T: int, dtype: str) -> np.ndarray:
    P, T_pad, hq_l, D = recv.shape
    out = torch.empty((T, P * hq_l, D), dtype=torch_dtype(dtype), device=DEV)
    out.view(torch.uint8).fill_(0x55)
    B.unpack_head2seq(t(recv, dtype), out)
    torch.cuda.synchronize()
    return B.to_host(out)


def new_cache(num_blocks: int, hkv_l: int, D: int, dtype: str, fill_byte: int = 0xA5) -> torch.Tensor:
    c = torch.empty((num_blocks, hkv_l, 2, 16 * D), dtype=torch_dtype(dtype), device=DEV)
    c.view(torch.uint8).fill_(fill_byte)
    return c


def new_cache_fp8(num_blocks: int, hkv_l: int, D: int, fill_byte: int = 0xA5) -> torch.Tensor:
    c = torch.empty((num_blocks, hkv_l, 2, 16 * D), dtype=torch.uint8, device=DEV)
    c.fill_(fill_byte)
    return c


def kv_write(cache: torch.Tensor, k_new: np.ndarray, v_new: np.ndarray, slots: np.ndarray, dtype: str,
             fp8_scales=(1.0, 1.0)) -> None:
    B.kv_write(t(k_new, dtype), t(v_new, dtype), ti(slots, np.int64), cache, fp8_scales[0], fp8_scales[1])
    torch.cuda.synchronize()


def cache_for_case(case, only_cached: bool = False, fill_byte: int = 0xA5, fp8_scales=None) -> torch.Tensor:
    """fp8_scales=(k_scale, v_scale): an FP8 E4M3 cache (uint8) instead of one in the case's type."""
    if fp8_scales is None:
        cache = new_cache(case.num_blocks, case.hkv_l, case.D, case.dtype, fill_byte)
    else:
        cache = new_cache_fp8(case.num_blocks, case.hkv_l, case.D, fill_byte)
    slots = case.slots
    if only_cached:
        slots = slots.copy()
        slots[case.new_token_index] = -1
    if case.k_ctx.shape[0]:
        kv_write(cache, case.k_ctx, case.v_ctx, slots, case.dtype, fp8_scales or (1.0, 1.0))
    return cache


def _scales(fp8_scales):
    return {} if fp8_scales is None else dict(k_scale=fp8_scales[0], v_scale=fp8_scales[1])


def prefill_case(case, cache: torch.Tensor, fused_new_kv: bool = False, fp8_scales=None) -> np.ndarray:
    """shiftattn_prefill on a workloads.AttnCase.  fused_new_kv: hand the new tokens' K/V to the call
    as strided views of one fused [total_q, hq_l + 2*hkv_l, D] buffer, the way an SP-mode caller would."""
    dt = case.dtype
    out = torch.empty((case.total_q, case.hq_l, case.D), dtype=torch_dtype(dt), device=DEV)
    kw = {}
    if fused_new_kv:
        fused = np.concatenate([case.q, case.k_ctx[case.new_token_index], case.v_ctx[case.new_token_index]], axis=1)
        ft = t(fused, dt)
        q = ft[:, :case.hq_l]
        kw = dict(k_new=ft[:, case.hq_l:case.hq_l + case.hkv_l], v_new=ft[:, case.hq_l + case.hkv_l:],
                  slot_mapping=ti(case.slots[case.new_token_index], np.int64))
    else:
        q = t(case.q, dt)
    B.prefill(q, cache, ti(case.block_table, np.int32), ti(case.cu_seqlens_q, np.int32), ti(case.ctx_lens, np.int32),
              int(case.q_lens.max()) if case.num_seqs else 0, int(case.ctx_lens.max()) if case.num_seqs else 0, out,
              case.softmax_scale, **kw, **_scales(fp8_scales))
    torch.cuda.synchronize()
    return B.to_host(out)


def decode_case(case, cache: torch.Tensor, fused_new_kv: bool = False, fp8_scales=None) -> np.ndarray:
    """shiftattn_decode on a case whose sequences all have one new token."""
    assert np.all(case.q_lens == 1)
    dt = case.dtype
    out = torch.empty((case.num_seqs, case.hq_l, case.D), dtype=torch_dtype(dt), device=DEV)
    kw = {}
    if fused_new_kv:
        fused = np.concatenate([case.q, case.k_ctx[case.new_token_index], case.v_ctx[case.new_token_index]], axis=1)
        ft = t(fused, dt)
        q = ft[:, :case.hq_l]
        kw = dict(k_new=ft[:, case.hq_l:case.hq_l + case.hkv_l], v_new=ft[:, case.hq_l + case.hkv_l:],
                  slot_mapping=ti(case.slots[case.new_token_index], np.int64))
    else:
        q = t(case.q, dt)
    B.decode(q, cache, ti(case.block_table, np.int32), ti(case.ctx_lens, np.int32),
             int(case.ctx_lens.max()) if case.num_seqs else 0, out, case.softmax_scale, **kw, **_scales(fp8_scales))
    torch.cuda.synchronize()
    return B.to_host(out)


def mixed_case(case, n_prefill: int, cache: torch.Tensor, fused_new_kv: bool = True, fp8_scales=None) -> np.ndarray:
    """shiftattn_mixed on a case whose first n_prefill sequences are chunks and whose others have one new token."""
    assert np.all(case.q_lens[n_prefill:] == 1)
    dt = case.dtype
    out = torch.empty((case.total_q, case.hq_l, case.D), dtype=torch_dtype(dt), device=DEV)
    kw = {}
    if fused_new_kv:
        fused = np.concatenate([case.q, case.k_ctx[case.new_token_index], case.v_ctx[case.new_token_index]], axis=1)
        ft = t(fused, dt)
        q = ft[:, :case.hq_l]
        kw = dict(k_new=ft[:, case.hq_l:case.hq_l + case.hkv_l], v_new=ft[:, case.hq_l + case.hkv_l:],
                  slot_mapping=ti(case.slots[case.new_token_index], np.int64))
    else:
        q = t(case.q, dt)
    pre_q, pre_ctx, dec_ctx = case.q_lens[:n_prefill], case.ctx_lens[:n_prefill], case.ctx_lens[n_prefill:]
    B.mixed(q, cache, ti(case.block_table, np.int32), ti(case.cu_seqlens_q[:n_prefill + 1], np.int32),
            ti(case.ctx_lens, np.int32), n_prefill, int(pre_q.max()) if n_prefill else 0,
            int(pre_ctx.max()) if n_prefill else 0, int(dec_ctx.max()) if len(dec_ctx) else 0, out, case.softmax_scale, **kw, **_scales(fp8_scales))
    torch.cuda.synchronize()
    return B.to_host(out)
