"""P virtual ranks on one host: the caller's side of Algorithm 1 around the attention path.

What a serving engine does *outside* the path under test, written with numpy slicing only:
cut the global fused-QKV activations [n, H + 2*H_kv, D] into the column slice a TP rank's
QKV projection would produce and the row slice an SP rank owns, and move send buffers between
members of an SP group.  The pack / unpack / KV-write / attention steps themselves are passed
in as a backend object (the CPU oracle in CPU tests, the HIP binding in GPU tests), so the same
scenario drives both.
"""
from __future__ import annotations

import numpy as np


def tp_column_slice(qkv: np.ndarray, H: int, H_kv: int, n_parts: int, part: int) -> np.ndarray:
    """Fused rows [n, h + 2*h_kv, D] that part `part` of an n_parts-way column (head) partition of
    the QKV projection produces: a contiguous run of query heads plus their GQA KV heads.  When
    there are fewer KV heads than parts, neighbouring parts recompute the same KV head (TP
    replicates KV weights, Sec. 3.2.1 'KV Cache Replication')."""
    h = H // n_parts
    q = qkv[:, part * h:(part + 1) * h]
    if H_kv >= n_parts:
        h_kv = H_kv // n_parts
        ks = slice(H + part * h_kv, H + (part + 1) * h_kv)
        vs = slice(H + H_kv + part * h_kv, H + H_kv + (part + 1) * h_kv)
    else:
        kv = (part * h) * H_kv // H          # GQA KV head of this part's first query head
        ks = slice(H + kv, H + kv + 1)
        vs = slice(H + H_kv + kv, H + H_kv + kv + 1)
    return np.ascontiguousarray(np.concatenate([q, qkv[:, ks], qkv[:, vs]], axis=1))


def local_heads(H: int, H_kv: int, n_parts: int):
    return H // n_parts, max(1, H_kv // n_parts)


def sp_mode_recv(backend, qkv: np.ndarray, H: int, H_kv: int, sp: int, tp: int, rank: int, dtype: str):
    """Fused rows [n_pad, hq_l + 2*hkv_l, D] that global rank `rank` holds after the first SP
    all-to-all of the base configuration (SP=sp, TP=tp).  Returns (recv, n_pad)."""
    n = qkv.shape[0]
    n_pad = -(-n // sp) * sp
    T = n_pad // sp
    t, r = rank % tp, rank // tp
    cols = tp_column_slice(qkv, H, H_kv, tp, t)               # this TP rank's heads, all rows
    h, h_kv = local_heads(H, H_kv, tp)
    sends = []
    for s in range(sp):                                        # members of this rank's SP group
        rows = cols[s * T:min((s + 1) * T, n)]                 # the last member may hold fewer real rows
        sends.append(backend.pack_seq2head(rows, sp, h, h_kv, T, dtype))
    recv = np.concatenate([snd[r] for snd in sends], axis=0)   # the exchange: pure data movement
    return recv, n_pad


def tp_mode_rows(qkv: np.ndarray, H: int, H_kv: int, sp: int, tp: int, rank: int, head_block) -> np.ndarray:
    """Fused rows the same global rank computes by itself in the shift configuration
    (SP=1, TP=sp*tp) when its weight shard follows the base configuration's head order."""
    return tp_column_slice(qkv, H, H_kv, sp * tp, head_block(sp, tp, rank))
