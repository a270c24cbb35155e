"""Seeded synthetic inputs for the head-shard attention path.

This module only draws numbers and lays out request metadata (context
lengths, block tables, slot lists).  It contains none of the method's
arithmetic: no attention, no packing, no cache layout.  Both the CPU oracle's
tests and the HIP path's tests/bench take their inputs from here, so the two
sides see identical bytes without sharing any code of the method itself.

Shapes follow the evaluation set-up of the paper (Table 4 head geometries,
Section 4.3 context sizes 2k-128k, chunked-prefill batches that mix prefill
chunks and decode tokens); the values are seeded Gaussians because the paper's
parameterised benchmarks use random request data (Section 4.1, Datasets iii).

Element types: "f32" arrays are numpy float32; "bf16" arrays are numpy uint16
holding bfloat16 bit patterns (fp32 rounded to nearest-even).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

BLOCK_SIZE = 16


# ----------------------------------------------------------------------------
# element helpers (storage only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest-even) and return the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a stored array to float64."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def elem_size(dtype: str) -> int:
    return {"bf16": 2, "f32": 4}[dtype]


def np_storage(dtype: str):
    return {"bf16": np.uint16, "f32": np.float32}[dtype]


def _gauss(rng: np.random.Generator, shape, dtype: str, scale: float) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


# ----------------------------------------------------------------------------
# attention cases
# ----------------------------------------------------------------------------
@dataclass
class AttnCase:
    """One batch for the attention entry points (local head shard of one GPU).

    Token order everywhere is sequence-major.  `k_ctx`/`v_ctx` hold every
    context token of every sequence (cached ones and new ones); the last
    `q_lens[s]` tokens of sequence s are the new tokens whose queries are in
    `q`.  `slots` gives the cache slot (block * block_size + offset) of each
    context token according to `block_table`.
    """

    name: str
    dtype: str
    hq_l: int
    hkv_l: int
    D: int
    block_size: int
    softmax_scale: float
    q_lens: np.ndarray           # int32 [S]
    ctx_lens: np.ndarray         # int32 [S]  (includes the new tokens)
    cu_seqlens_q: np.ndarray     # int32 [S+1]
    cu_ctx: np.ndarray           # int64 [S+1]
    q: np.ndarray                # [sum q_lens, hq_l, D]
    k_ctx: np.ndarray            # [sum ctx_lens, hkv_l, D]
    v_ctx: np.ndarray            # [sum ctx_lens, hkv_l, D]
    block_table: np.ndarray      # int32 [S, max_blocks_per_seq], unused = -1
    num_blocks: int
    slots: np.ndarray            # int64 [sum ctx_lens]
    new_token_index: np.ndarray  # int64 [sum q_lens] index into k_ctx rows

    @property
    def num_seqs(self) -> int:
        return int(self.q_lens.shape[0])

    @property
    def total_q(self) -> int:
        return int(self.cu_seqlens_q[-1])

    @property
    def max_blocks_per_seq(self) -> int:
        return int(self.block_table.shape[1])

    def causal_pairs(self) -> int:
        """(query, visible key) pairs per query head, for the flop convention."""
        q = self.q_lens.astype(np.int64)
        c = self.ctx_lens.astype(np.int64)
        return int(np.sum(q * (c - q) + q * (q + 1) // 2))

    def flops(self) -> int:
        """4*D per visible pair per query head (QK^T and PV; masked pairs excluded)."""
        return 4 * self.D * self.hq_l * self.causal_pairs()

    def kv_bytes(self) -> int:
        """K and V bytes of all context tokens, read once per (sequence, KV head)."""
        return int(self.ctx_lens.astype(np.int64).sum()) * 2 * self.hkv_l * self.D * elem_size(self.dtype)


def make_attn_case(
    name: str,
    seed: int,
    dtype: str,
    seqs: Sequence[Tuple[int, int]],
    hq_l: int,
    hkv_l: int,
    D: int,
    *,
    value_scale: float = 1.0,
    pool_factor: float = 2.0,
    permute_blocks: bool = True,
    block_size: int = BLOCK_SIZE,
    softmax_scale: float | None = None,
    min_pool_blocks: int = 0,
) -> AttnCase:
    """Draw one batch.  `seqs` lists (q_len, ctx_len) per sequence, ctx_len >= q_len."""
    rng = np.random.Generator(np.random.PCG64(seed))
    q_lens = np.array([s[0] for s in seqs], dtype=np.int32)
    ctx_lens = np.array([s[1] for s in seqs], dtype=np.int32)
    assert np.all(ctx_lens >= q_lens) and np.all(q_lens >= 0)
    S = len(seqs)
    cu_q = np.zeros(S + 1, dtype=np.int32)
    cu_q[1:] = np.cumsum(q_lens)
    cu_c = np.zeros(S + 1, dtype=np.int64)
    cu_c[1:] = np.cumsum(ctx_lens.astype(np.int64))
    total_q, total_c = int(cu_q[-1]), int(cu_c[-1])

    q = _gauss(rng, (total_q, hq_l, D), dtype, value_scale)
    k = _gauss(rng, (total_c, hkv_l, D), dtype, value_scale)
    v = _gauss(rng, (total_c, hkv_l, D), dtype, value_scale)

    blocks_per_seq = (ctx_lens.astype(np.int64) + block_size - 1) // block_size
    used = int(blocks_per_seq.sum())
    num_blocks = max(int(np.ceil(used * pool_factor)), used, 1, min_pool_blocks)
    if permute_blocks:
        ids = rng.permutation(num_blocks)[:used].astype(np.int32)
    else:
        ids = np.arange(used, dtype=np.int32)
    max_blocks = max(int(blocks_per_seq.max()) if S else 1, 1)
    table = np.full((S, max_blocks), -1, dtype=np.int32)
    slots = np.empty(total_c, dtype=np.int64)
    new_idx = np.empty(total_q, dtype=np.int64)
    at = 0
    for s in range(S):
        nb = int(blocks_per_seq[s])
        table[s, :nb] = ids[at:at + nb]
        at += nb
        t = np.arange(int(ctx_lens[s]), dtype=np.int64)
        slots[cu_c[s]:cu_c[s + 1]] = table[s, t // block_size].astype(np.int64) * block_size + t % block_size
        ql = int(q_lens[s])
        new_idx[cu_q[s]:cu_q[s + 1]] = cu_c[s + 1] - ql + np.arange(ql, dtype=np.int64)
    if softmax_scale is None:
        softmax_scale = 1.0 / float(np.sqrt(D))
    return AttnCase(name, dtype, hq_l, hkv_l, D, block_size, float(softmax_scale), q_lens, ctx_lens,
                    cu_q, cu_c, q, k, v, table, num_blocks, slots, new_idx)


# ----------------------------------------------------------------------------
# sequence<->head exchange cases
# ----------------------------------------------------------------------------
@dataclass
class XchgCase:
    """Input of the send-side pack: one SP rank's rows of the fused QKV activations."""

    name: str
    dtype: str
    P: int
    h: int        # query heads on the source side of the exchange
    h_kv: int     # KV heads on the source side (0: query-only rows)
    D: int
    T: int        # real rows held by this rank
    T_pad: int    # rows per send buffer (>= T)
    x: np.ndarray  # [T, h + 2*h_kv, D]

    def bytes_moved(self) -> int:
        """Input read once plus output written once."""
        e = elem_size(self.dtype)
        hq_l = self.h // self.P
        hkv_l = 0 if self.h_kv == 0 else max(1, self.h_kv // self.P)
        rd = self.T * (self.h + 2 * self.h_kv) * self.D * e
        wr = self.P * self.T_pad * (hq_l + 2 * hkv_l) * self.D * e
        return rd + wr


def make_xchg_case(name: str, seed: int, dtype: str, P: int, h: int, h_kv: int, D: int, T: int,
                   T_pad: int | None = None, value_scale: float = 1.0) -> XchgCase:
    rng = np.random.Generator(np.random.PCG64(seed))
    x = _gauss(rng, (T, h + 2 * h_kv, D), dtype, value_scale)
    return XchgCase(name, dtype, P, h, h_kv, D, T, T if T_pad is None else T_pad, x)


# ----------------------------------------------------------------------------
# the five named configurations (seed = configuration number)
# ----------------------------------------------------------------------------
def config1_attn() -> AttnCase:
    """Tiny fp32 shard: one 256-token causal prefill, 4 query heads / 1 KV head, head_dim 64."""
    return make_attn_case("cfg1_tiny_f32", 1, "f32", [(256, 256)], 4, 1, 64, permute_blocks=False,
                          pool_factor=1.0)


def config1_xchg() -> XchgCase:
    """Query-only hidden [256, 8 heads, 64] fp32 exchanged at P=2."""
    return make_xchg_case("cfg1_xchg", 1, "f32", 2, 8, 0, 64, 256)


def config2_attn(data_scaled: bool = False, n_seqs: int = 4, seq_len: int = 4096) -> AttnCase:
    """8B-shaped shard at P=8: bf16, 4 query / 1 KV head, head_dim 128, 4 x 4096 causal prefill,
    paged KV in a random permutation of a pool twice the used size.

    data_scaled=False: values N(0,1), logits ~ N(0,1) after the 1/sqrt(D) softmax scale.
    data_scaled=True : values N(0,1)/sqrt(128) as the configuration text can also be read."""
    vs = 1.0 / float(np.sqrt(128.0)) if data_scaled else 1.0
    return make_attn_case("cfg2_8b_prefill", 2, "bf16", [(seq_len, seq_len)] * n_seqs, 4, 1, 128,
                          value_scale=vs, pool_factor=2.0)


def config3_attn(seq_len: int = 16384) -> AttnCase:
    """70B-shaped shard at P=8: bf16, 8 query / 1 KV head, one 16384-token causal prefill."""
    return make_attn_case("cfg3_70b_prefill", 3, "bf16", [(seq_len, seq_len)], 8, 1, 128, pool_factor=2.0)


def config3_xchg(T: int = 16384) -> XchgCase:
    """Query-only hidden [16384, 64 heads, 128] bf16 packed into 8 send buffers."""
    return make_xchg_case("cfg3_xchg", 3, "bf16", 8, 64, 0, 128, T)


def config4_attn(n_seqs: int = 256, lo: int = 512, hi: int = 8192) -> AttnCase:
    """Batch decode, 70B shard: 256 sequences, 1 query token each, contexts uniform in [512, 8192]."""
    rng = np.random.Generator(np.random.PCG64(4))
    ctx = rng.integers(lo, hi + 1, size=n_seqs)
    return make_attn_case("cfg4_70b_decode", 4, "bf16", [(1, int(c)) for c in ctx], 8, 1, 128,
                          pool_factor=1.25)


def config5_attn(chunk: int = 2048, cached: int = 131072, n_dec: int = 64, lo: int = 1024,
                 hi: int = 32768) -> Tuple[AttnCase, int]:
    """Mixed long-context step, 70B shard: one chunked prefill (2048 new tokens continuing a
    131072-token cached context) plus 64 decode sequences with contexts uniform in [1024, 32768],
    all in one shared block pool.  Returns (case, number_of_prefill_sequences); sequence 0 is the
    prefill chunk, the rest are decodes."""
    rng = np.random.Generator(np.random.PCG64(5))
    ctx = rng.integers(lo, hi + 1, size=n_dec)
    seqs = [(chunk, cached + chunk)] + [(1, int(c)) for c in ctx]
    return make_attn_case("cfg5_mixed", 5, "bf16", seqs, 8, 1, 128, pool_factor=1.1), 1


def sub_case(case: AttnCase, seq_ids: Sequence[int], name: str | None = None) -> AttnCase:
    """View of a subset of sequences sharing the parent's block pool (same slots, same cache)."""
    seq_ids = list(seq_ids)
    q_lens = case.q_lens[seq_ids]
    ctx_lens = case.ctx_lens[seq_ids]
    cu_q = np.zeros(len(seq_ids) + 1, dtype=np.int32)
    cu_q[1:] = np.cumsum(q_lens)
    cu_c = np.zeros(len(seq_ids) + 1, dtype=np.int64)
    cu_c[1:] = np.cumsum(ctx_lens.astype(np.int64))
    q = np.concatenate([case.q[case.cu_seqlens_q[s]:case.cu_seqlens_q[s + 1]] for s in seq_ids], axis=0)
    k = np.concatenate([case.k_ctx[case.cu_ctx[s]:case.cu_ctx[s + 1]] for s in seq_ids], axis=0)
    v = np.concatenate([case.v_ctx[case.cu_ctx[s]:case.cu_ctx[s + 1]] for s in seq_ids], axis=0)
    slots = np.concatenate([case.slots[case.cu_ctx[s]:case.cu_ctx[s + 1]] for s in seq_ids], axis=0)
    new_idx = np.concatenate(
        [cu_c[i + 1] - int(q_lens[i]) + np.arange(int(q_lens[i]), dtype=np.int64) for i in range(len(seq_ids))]
        or [np.zeros(0, dtype=np.int64)])
    nb = (ctx_lens.astype(np.int64) + case.block_size - 1) // case.block_size
    mb = max(int(nb.max()) if len(seq_ids) else 1, 1)
    table = np.ascontiguousarray(case.block_table[seq_ids][:, :mb])
    return AttnCase(name or case.name + "_sub", case.dtype, case.hq_l, case.hkv_l, case.D, case.block_size,
                    case.softmax_scale, q_lens, ctx_lens, cu_q, cu_c, q, k, v, table, case.num_blocks,
                    slots, new_idx)
