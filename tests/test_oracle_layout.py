"""Pins for the oracle's layout steps: pack, exchange, unpack, KV write, rank -> head map (no GPU).

Pinned against the paper's printed examples (tests/golden), against direct numpy slicing of
the global tensor, and against attention-level invariants: if the pack sent a wrong head, a
wrong KV replica or a wrong row anywhere, sharded attention would stop matching unsharded
attention, and the TP-written cache would stop matching the SP-written cache.
"""
import ast
import os

import numpy as np
import pytest

import virtual_ranks as VR
from paper_2509_16495_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split("=", 1)
            out[k.strip()] = ast.literal_eval(v.strip())
    return out


def test_paper_process_groups_example(oracle):
    g = _read_golden("process_groups_sp3_tp2.txt")
    sp, tp = g["SP"], g["TP"]
    tp_groups, sp_groups, sp_tp = oracle.process_groups(sp, tp)
    assert tp_groups == g["TP_GROUPS"] and sp_groups == g["SP_GROUPS"] and sp_tp == g["SP_TP_GROUP"]
    for rank, head in g["HEAD_OF_RANK"].items():
        assert oracle.head_block(sp, tp, rank) == head
    # listing ranks by the head block they hold reproduces the interleaved order of Sec. 3.3.1
    blocks = [oracle.head_block(sp, tp, r) for r in range(sp * tp)]
    assert sorted(blocks) == list(range(sp * tp))
    assert [blocks.index(b) for b in range(sp * tp)] == g["INTERLEAVED_ORDER"] == sp_tp[0]
    # pure TP (sp=1) and pure SP (tp=1) keep the natural order
    assert [oracle.head_block(1, 6, r) for r in range(6)] == list(range(6))
    assert [oracle.head_block(6, 1, r) for r in range(6)] == list(range(6))


def test_paper_padding_and_replication_examples(oracle):
    g = _read_golden("padding_and_replication.txt")
    n, sp = g["BATCH"], g["SP"]
    # unpadded: ceil split leaves one rank with 2 tokens while the average is 9/8
    assert -(-n // sp) == g["UNPADDED_MAX_TOKENS_PER_RANK"]
    # padded pack: every rank sends buffers of T = n_pad/SP rows; here n_pad = 16, T = 2
    n_pad = -(-n // sp) * sp
    assert n_pad == 16 and n_pad // sp == 2
    x = W.make_xchg_case("t", 31, "f32", sp, 8, 8, 4, T=1, T_pad=2).x
    send = oracle.pack_seq2head(x, sp, 8, 8, 2, "f32")
    assert send.shape == (8, 2, 3, 4) and np.all(send[:, 1] == 0) and not np.any(send[:, 0] == 0)
    # replication: 32 q / 4 kv heads over 8 ranks -> rank r gets kv head r // 2, q heads [4r, 4r+4)
    P, h, h_kv = g["RANKS"], g["Q_HEADS"], g["KV_HEADS"]
    assert [oracle.kv_head_of_block(p, P, h_kv) for p in range(P)] == [0, 0, 1, 1, 2, 2, 3, 3]
    x = W.make_xchg_case("t", 32, "bf16", P, h, h_kv, 8, T=5).x
    send = oracle.pack_seq2head(x, P, h, h_kv, 5, "bf16")
    assert send.shape == (P, 5, 4 + 2, 8)
    for p in range(P):
        assert np.array_equal(send[p][:, :4], x[:, 4 * p:4 * p + 4])
        assert np.array_equal(send[p][:, 4], x[:, h + p // 2])
        assert np.array_equal(send[p][:, 5], x[:, h + h_kv + p // 2])
    assert 1.0 / 8 == g["SHIFT_OVERHEAD_AT_SP8"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("P,h,h_kv,T,T_pad", [(2, 8, 0, 256, 256), (4, 8, 4, 7, 9), (8, 16, 2, 5, 5),
                                              (2, 8, 4, 0, 3), (1, 3, 1, 4, 4), (3, 6, 6, 10, 11)])
def test_pack_equals_direct_slicing(oracle, dtype, P, h, h_kv, T, T_pad):
    x = W.make_xchg_case("t", 33, dtype, P, h, h_kv, 16, T, T_pad).x
    send = oracle.pack_seq2head(x, P, h, h_kv, T_pad, dtype)
    hq_l = h // P
    hkv_l = oracle.local_kv_heads(P, h_kv)
    assert send.shape == (P, T_pad, hq_l + 2 * hkv_l, 16)
    assert not np.any(send[:, T:].view(np.uint8))                      # pad rows are zero bytes
    for p in range(P):
        want = VR.tp_column_slice(x, h, h_kv, P, p) if h_kv else x[:, p * hq_l:(p + 1) * hq_l]
        assert np.array_equal(send[p][:T], want)


def test_pack_exchange_unpack_roundtrip(oracle):
    """Query-only hidden rows through pack -> all-to-all -> (identity attention) -> all-to-all ->
    unpack come back unchanged on every rank (Algorithm 1 shape algebra:
    [n/SP, h] -> [n, h/SP] -> [n/SP, h])."""
    P, h, D, n = 4, 8, 16, 22
    n_pad = -(-n // P) * P
    T = n_pad // P
    hidden = W.make_xchg_case("t", 34, "bf16", P, h, 0, D, n).x
    real = [max(0, min(T, n - s * T)) for s in range(P)]
    sends = [oracle.pack_seq2head(hidden[s * T:s * T + real[s]], P, h, 0, T, "bf16") for s in range(P)]
    recvs = [oracle.exchange(sends, r) for r in range(P)]              # [n_pad, h/P, D] on rank r
    for r in range(P):
        assert recvs[r].shape == (n_pad, h // P, D)
        assert np.array_equal(recvs[r][:n], hidden[:, r * 2:(r + 1) * 2])
    # second all-to-all: rank r sends row slice s of its attention output to rank s
    for s in range(P):
        back = np.stack([recvs[r][s * T:(s + 1) * T] for r in range(P)])      # recv[P][T, h/P, D]
        out = oracle.unpack_head2seq(back, real[s], "bf16")
        assert np.array_equal(out, hidden[s * T:s * T + real[s]])


def test_kv_write_places_rows_and_keeps_sentinel(oracle):
    case = W.make_attn_case("t", 35, "bf16", [(5, 37), (1, 16)], 4, 2, 8, pool_factor=3.0)
    cache = oracle.new_cache(case.num_blocks, 2, 16, 8, "bf16", 0xA5)
    slots = case.slots.copy()
    slots[3] = -1                                                      # a padding row
    oracle.kv_write(cache, case.k_ctx, case.v_ctx, slots, 16, "bf16")
    touched = np.zeros(cache.shape, dtype=bool)
    for i, slot in enumerate(slots):
        if slot < 0:
            continue
        blk, off = divmod(int(slot), 16)
        for g in range(2):
            assert np.array_equal(cache[blk, g, 0].reshape(16, 8)[off], case.k_ctx[i, g])      # K token-major
            assert np.array_equal(cache[blk, g, 1].reshape(8, 16)[:, off], case.v_ctx[i, g])   # V dim-major
            touched[blk, g, 0].reshape(16, 8)[off] = True
            touched[blk, g, 1].reshape(8, 16)[:, off] = True
    assert np.all(cache[~touched] == 0xA5A5)


@pytest.mark.parametrize("sp,tp,H,H_kv", [(3, 2, 12, 6), (2, 2, 8, 2), (8, 1, 32, 4), (4, 2, 16, 8), (1, 4, 8, 4)])
def test_sp_cache_equals_tp_cache_and_shards_equal_unsharded(oracle, sp, tp, H, H_kv):
    """KV cache invariance (Sec. 3.1, 3.3.1): on every rank the cache written from rows that came
    through the SP exchange is byte-identical to the cache written from the rank's own shift-config
    (full TP) rows, and attention over the shards, reassembled by head block, is unsharded attention."""
    D, B, dtype = 16, 16, "bf16"
    P = sp * tp
    whole = W.make_attn_case("t", 36, dtype, [(11, 30), (1, 20), (7, 7)], H, H_kv, D, pool_factor=1.5)
    n = whole.total_q
    qkv = np.concatenate([whole.q, whole.k_ctx[whole.new_token_index], whole.v_ctx[whole.new_token_index]], axis=1)
    ref_cache = oracle.cache_for_case(whole)
    ref_out = oracle.attention_case(whole, ref_cache)
    hq_l, hkv_l = VR.local_heads(H, H_kv, P)
    new_slots = whole.slots[whole.new_token_index]
    for rank in range(P):
        b = oracle.head_block(sp, tp, rank)
        # cached context of this rank's KV heads (written earlier, identical in both modes)
        kv0 = (b * hq_l) * H_kv // H
        k_old, v_old = whole.k_ctx[:, kv0:kv0 + hkv_l], whole.v_ctx[:, kv0:kv0 + hkv_l]
        old_slots = whole.slots.copy()
        old_slots[whole.new_token_index] = -1
        caches = []
        for mode in ("sp", "tp"):
            cache = oracle.new_cache(whole.num_blocks, hkv_l, B, D, dtype)
            oracle.kv_write(cache, k_old, v_old, old_slots, B, dtype)
            if mode == "sp":
                rows, n_pad = VR.sp_mode_recv(oracle, qkv, H, H_kv, sp, tp, rank, dtype)
            else:
                rows, n_pad = VR.tp_mode_rows(qkv, H, H_kv, sp, tp, rank, oracle.head_block), n
            slots = np.full(n_pad, -1, dtype=np.int64)
            slots[:n] = new_slots
            k_new, v_new = rows[:, hq_l:hq_l + hkv_l], rows[:, hq_l + hkv_l:]
            oracle.kv_write(cache, k_new, v_new, slots[:rows.shape[0]], B, dtype)
            caches.append((cache, rows))
        assert caches[0][0].tobytes() == caches[1][0].tobytes()
        assert np.array_equal(caches[0][1][:n], caches[1][1])
        shard = W.sub_case(whole, range(whole.num_seqs))
        shard.hq_l, shard.hkv_l = hq_l, hkv_l
        shard.q = np.ascontiguousarray(caches[0][1][:n, :hq_l])
        out = oracle.attention_case(shard, caches[0][0])
        assert np.array_equal(out, ref_out[:, b * hq_l:(b + 1) * hq_l])
