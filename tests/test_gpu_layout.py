"""GPU parity of the data-movement steps against the CPU oracle: bit-exact, through the C ABI."""
import numpy as np
import pytest

import virtual_ranks as VR
from paper_2509_16495_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_backend
    return gpu_backend


XCHG_CASES = [
    # dtype, P, h, h_kv, D, T, T_pad
    ("f32", 2, 8, 0, 64, 256, 256),      # the tiny configuration's exchange
    ("bf16", 8, 64, 8, 128, 300, 300),   # fused q|k|v rows of a 70B-shaped layer, ragged tail of the launch
    ("bf16", 8, 32, 4, 128, 65, 70),     # fewer KV heads than ranks: replication inside the send buffers
    ("bf16", 4, 40, 8, 128, 33, 40),     # five query heads per KV head
    ("f32", 3, 6, 6, 8, 10, 11),
    ("bf16", 2, 8, 4, 64, 0, 3),         # a rank that holds padding rows only
    ("bf16", 1, 3, 1, 8, 4, 4),
    ("bf16", 8, 64, 0, 128, 1031, 1031),
]


@pytest.mark.parametrize("dtype,P,h,h_kv,D,T,T_pad", XCHG_CASES)
def test_pack_bit_exact(oracle, G, dtype, P, h, h_kv, D, T, T_pad):
    x = W.make_xchg_case("t", 41, dtype, P, h, h_kv, D, T, T_pad).x
    want = oracle.pack_seq2head(x, P, h, h_kv, T_pad, dtype)
    got = G.pack_seq2head(x, P, h, h_kv, T_pad, dtype)
    assert got.tobytes() == want.tobytes()


@pytest.mark.parametrize("dtype,P,h,h_kv,D,T,T_pad", XCHG_CASES)
def test_unpack_bit_exact(oracle, G, dtype, P, h, h_kv, D, T, T_pad):
    recv = W.make_xchg_case("t", 42, dtype, 1, h // P, 0, D, P * T_pad).x.reshape(P, T_pad, h // P, D)
    want = oracle.unpack_head2seq(recv, T, dtype)
    got = G.unpack_head2seq(recv, T, dtype)
    assert got.shape == (T, h, D) and got.tobytes() == want.tobytes()


def test_pack_unpack_full_size_70b_hidden(oracle, G):
    """The benchmarked exchange: hidden [16384, 64 heads, 128] bf16 into 8 send buffers and back."""
    c = W.config3_xchg()
    want = oracle.pack_seq2head(c.x, c.P, c.h, c.h_kv, c.T_pad, c.dtype)
    got = G.pack_seq2head(c.x, c.P, c.h, c.h_kv, c.T_pad, c.dtype)
    assert got.tobytes() == want.tobytes()
    back = G.unpack_head2seq(got, c.T, c.dtype)
    assert back.tobytes() == c.x.tobytes() == oracle.unpack_head2seq(want, c.T, c.dtype).tobytes()


@pytest.mark.parametrize("dtype,hkv_l,D", [("bf16", 1, 128), ("bf16", 2, 64), ("f32", 1, 64), ("f32", 3, 8)])
def test_kv_write_bit_exact(oracle, G, dtype, hkv_l, D):
    case = W.make_attn_case("t", 43, dtype, [(40, 300), (1, 17), (16, 16), (0, 5)], hkv_l, hkv_l, D, pool_factor=1.7)
    slots = case.slots.copy()
    slots[::7] = -1                                   # padding rows scattered through the batch
    want = oracle.new_cache(case.num_blocks, hkv_l, 16, D, dtype)
    oracle.kv_write(want, case.k_ctx, case.v_ctx, slots, 16, dtype)
    cache = G.new_cache(case.num_blocks, hkv_l, D, dtype)
    G.kv_write(cache, case.k_ctx, case.v_ctx, slots, dtype)
    from paper_2509_16495_amd import binding as B
    assert B.to_host(cache).tobytes() == want.tobytes()


@pytest.mark.parametrize("hkv_l", [1, 2])
def test_kv_write_whole_blocks_and_ragged_runs(oracle, G, hkv_l):
    """bf16, D=128: the writer works run by run (consecutive tokens in consecutive slots of one block): whole
    blocks, runs that start or end inside a block, a padding row inside a run, the tail of the batch; untouched
    slots keep their bytes."""
    from paper_2509_16495_amd import binding as B
    case = W.make_attn_case("t", 45, "bf16", [(64, 64), (32, 160), (16, 21), (48, 48), (5, 5)], hkv_l, hkv_l, 128,
                            pool_factor=1.4)
    for holes in ((), (3,), (70, 71, 120)):
        slots = case.slots[case.new_token_index].copy()
        slots[list(holes)] = -1
        k, v = case.k_ctx[case.new_token_index], case.v_ctx[case.new_token_index]
        want = oracle.new_cache(case.num_blocks, hkv_l, 16, 128, "bf16", fill_byte=0x7F)   # untouched slots keep it
        oracle.kv_write(want, k, v, slots, 16, "bf16")
        cache = G.new_cache(case.num_blocks, hkv_l, 128, "bf16", fill_byte=0x7F)
        G.kv_write(cache, k, v, slots, "bf16")
        assert B.to_host(cache).tobytes() == want.tobytes()


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("seed", [46, 47, 48])
def test_kv_write_arbitrary_slot_patterns(oracle, G, seed, fp8):
    """bf16, D=128, slot patterns a serving engine can produce in one batch, in random order: runs of every length
    1..16 at every offset inside a block, runs that continue into another block, single tokens, padding rows, slots
    that descend, a batch size that is no multiple of 16.  Every slot is used at most once; bit-exact cache."""
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(seed))
    hkv_l, D, n_blocks = 2, 128, 400
    free = list(rng.permutation(n_blocks))
    pieces = []
    for _ in range(150):
        kind = rng.integers(0, 5)
        if kind == 0:                                   # a run inside one block
            off = int(rng.integers(0, 16)); ln = int(rng.integers(1, 17 - off))
            pieces.append(free.pop() * 16 + off + np.arange(ln))
        elif kind == 1:                                 # a sequence stretch over several blocks, starting anywhere
            off = int(rng.integers(0, 16)); ln = int(rng.integers(1, 70))
            pos = off + np.arange(ln)
            blocks = [free.pop() for _ in range(pos[-1] // 16 + 1)]
            pieces.append(np.array([blocks[q // 16] * 16 + q % 16 for q in pos]))
        elif kind == 2:                                 # padding rows
            pieces.append(np.full(int(rng.integers(1, 4)), -1))
        elif kind == 3:                                 # single decode tokens
            pieces.append(np.array([free.pop() * 16 + int(rng.integers(0, 16)) for _ in range(int(rng.integers(1, 6)))]))
        else:                                           # consecutive slots in descending order
            off = int(rng.integers(0, 12)); ln = int(rng.integers(2, 17 - off))
            pieces.append(free.pop() * 16 + off + np.arange(ln)[::-1])
    slots = np.concatenate(pieces).astype(np.int64)
    n = len(slots)
    assert n % 16 != 0
    used = slots[slots >= 0]
    assert len(np.unique(used)) == len(used)
    k = W.f32_to_bf16_bits(rng.standard_normal((n, hkv_l, D), dtype=np.float32))
    v = W.f32_to_bf16_bits(rng.standard_normal((n, hkv_l, D), dtype=np.float32))
    if fp8:   # the quantising writer: codes of x / scale, a scale that is no power of two
        ks, vs = 0.037, 0.021
        want = oracle.new_cache(n_blocks, hkv_l, 16, D, "fp8_e4m3", fill_byte=0x7F)
        oracle.kv_write_fp8(want, k, v, slots, 16, "bf16", ks, vs)
        cache = G.new_cache_fp8(n_blocks, hkv_l, D, fill_byte=0x7F)
        G.kv_write(cache, k, v, slots, "bf16", fp8_scales=(ks, vs))
    else:
        want = oracle.new_cache(n_blocks, hkv_l, 16, D, "bf16", fill_byte=0x7F)
        oracle.kv_write(want, k, v, slots, 16, "bf16")
        cache = G.new_cache(n_blocks, hkv_l, D, "bf16", fill_byte=0x7F)
        G.kv_write(cache, k, v, slots, "bf16")
    assert B.to_host(cache).tobytes() == want.tobytes()


@pytest.mark.parametrize("sp,tp,H,H_kv", [(3, 2, 12, 6), (8, 1, 32, 4), (4, 2, 16, 8), (4, 2, 40, 8)])
def test_sp_cache_equals_tp_cache_on_gpu(oracle, G, sp, tp, H, H_kv):
    """KV-cache invariance through the GPU kernels: pack -> exchange -> fused KV write in SP mode
    leaves exactly the bytes that the direct TP-mode write leaves, and both equal the oracle's cache."""
    from paper_2509_16495_amd import binding as B
    D, dtype = 64, "bf16"
    P = sp * tp
    whole = W.make_attn_case("t", 44, dtype, [(37, 90), (1, 33), (20, 20)], H, H_kv, D, pool_factor=1.5)
    n = whole.total_q
    qkv = np.concatenate([whole.q, whole.k_ctx[whole.new_token_index], whole.v_ctx[whole.new_token_index]], axis=1)
    hq_l, hkv_l = VR.local_heads(H, H_kv, P)
    old_slots = whole.slots.copy()
    old_slots[whole.new_token_index] = -1
    for rank in range(P):
        b = oracle.head_block(sp, tp, rank)
        assert B.head_block(sp, tp, rank) == b
        kv0 = (b * hq_l) * H_kv // H
        k_old, v_old = whole.k_ctx[:, kv0:kv0 + hkv_l], whole.v_ctx[:, kv0:kv0 + hkv_l]
        images = []
        for mode in ("sp", "tp"):
            cache = G.new_cache(whole.num_blocks, hkv_l, D, dtype)
            G.kv_write(cache, k_old, v_old, old_slots, dtype)
            if mode == "sp":
                rows, n_pad = VR.sp_mode_recv(G, qkv, H, H_kv, sp, tp, rank, dtype)
            else:
                rows, n_pad = VR.tp_mode_rows(qkv, H, H_kv, sp, tp, rank, B.head_block), n
            slots = np.full(n_pad, -1, dtype=np.int64)
            slots[:n] = whole.slots[whole.new_token_index]
            fused = G.t(rows, dtype)                                   # K/V written from views of the fused rows
            B.kv_write(fused[:, hq_l:hq_l + hkv_l], fused[:, hq_l + hkv_l:], G.ti(slots, np.int64), cache)
            images.append(B.to_host(cache).tobytes())
        want = oracle.new_cache(whole.num_blocks, hkv_l, 16, D, dtype)
        oracle.kv_write(want, k_old, v_old, old_slots, 16, dtype)
        oracle.kv_write(want, whole.k_ctx[whole.new_token_index][:, kv0:kv0 + hkv_l],
                        whole.v_ctx[whole.new_token_index][:, kv0:kv0 + hkv_l], whole.slots[whole.new_token_index], 16, dtype)
        assert images[0] == images[1] == want.tobytes()
