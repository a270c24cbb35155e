"""GPU parity of prefill and decode attention against the CPU fp64 oracle, through the C ABI.

Tolerances (absolute, on outputs of O(1) magnitude):
  bf16 tensors, fp32 accumulation : max |err| <= 2e-2 and mean |err| <= 1e-3
  fp32 tensors                    : max |err| <= 1e-5
and, where outputs are tiny (values pre-scaled by 1/sqrt(128)), additionally max |err| <= 2e-2 * max |ref|.
Small cases are compared element by element; the benchmark-sized configurations on sampled rows
(all heads of every sampled token) that the oracle can afford.
"""
import os

import numpy as np
import pytest

from paper_2509_16495_amd import workloads as W

pytestmark = pytest.mark.gpu

BF16_MAX, BF16_MEAN, F32_MAX = 2e-2, 1e-3, 1e-5


@pytest.fixture(scope="module")
def G():
    import gpu_backend
    return gpu_backend


def _check(got_bits, want, dtype, relative=False):
    got = W.to_f64(got_bits, dtype)
    assert got.shape == want.shape
    assert np.all(np.isfinite(got))
    err = np.abs(got - want)
    if dtype == "f32":
        assert err.max() <= F32_MAX, err.max()
    else:
        assert err.max() <= BF16_MAX and err.mean() <= BF16_MEAN, (err.max(), err.mean())
        if relative:
            assert err.max() <= BF16_MAX * np.abs(want).max(), (err.max(), np.abs(want).max())


def _sample_rows(case, n_random, seed, edge=32):
    """Sampled query tokens: the first and last `edge` tokens of every sequence plus random ones."""
    rng = np.random.default_rng(seed)
    rows = []
    for s in range(case.num_seqs):
        a, b = int(case.cu_seqlens_q[s]), int(case.cu_seqlens_q[s + 1])
        rows += list(range(a, min(a + edge, b))) + list(range(max(a, b - edge), b))
    rows += list(rng.integers(0, case.total_q, size=n_random))
    return np.unique(np.array(rows, dtype=np.int64))


# ------------------------------------------------------------------------------------------------------
# small cases, element by element
# ------------------------------------------------------------------------------------------------------
def test_config1_tiny_fp32_prefill(oracle, G):
    case = W.config1_attn()
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    got = G.prefill_case(case, G.cache_for_case(case))
    _check(got, want, "f32")


PREFILL_SMALL = [
    # seqs (q_len, ctx), hq_l, hkv_l  - bf16, D=128 (MFMA path)
    ([(200, 200), (77, 300), (1, 50), (130, 130)], 8, 1),   # several tiles, ragged tails, chunked, one decode-like row
    ([(64, 64), (33, 33), (16, 16)], 4, 1),
    ([(150, 150), (5, 260)], 8, 2),                          # two KV heads
    ([(100, 100)], 4, 4),                                    # no GQA sharing
    ([(90, 190)], 6, 2),                                     # three query heads per KV head (not a power of two)
    ([(300, 300)], 16, 1),
    ([(0, 10), (40, 40), (0, 0)], 4, 1),                     # empty chunks in the batch
    ([(140, 140), (31, 333)], 5, 1),                         # 40q/8kv model on 8 ranks (Table 4, Llama-17B-16E): 5 per KV head
    ([(129, 200)], 10, 2),                                   # the same model on 4 ranks
]


@pytest.mark.parametrize("seqs,hq_l,hkv_l", PREFILL_SMALL)
def test_prefill_bf16_small(oracle, G, seqs, hq_l, hkv_l):
    case = W.make_attn_case("t", 51, "bf16", seqs, hq_l, hkv_l, 128)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    got = G.prefill_case(case, G.cache_for_case(case))
    _check(got, want, "bf16")


def test_prefill_fused_kv_write_from_strided_views(oracle, G):
    """New tokens' K/V arrive with the call as views into a fused receive buffer; the cache afterwards
    and the attention output both match 'write, then attend'."""
    from paper_2509_16495_amd import binding as B
    case = W.make_attn_case("t", 52, "bf16", [(70, 170), (128, 128), (1, 40)], 8, 1, 128)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    cache = G.cache_for_case(case, only_cached=True)
    got = G.prefill_case(case, cache, fused_new_kv=True)
    _check(got, want, "bf16")
    assert B.to_host(cache).tobytes() == oracle.cache_for_case(case).tobytes()


def test_prefill_split_over_keys(oracle, G):
    """A short chunk on a long cached context is split into key ranges and merged."""
    from paper_2509_16495_amd import binding as B
    case = W.make_attn_case("t", 53, "bf16", [(48, 9000)], 8, 1, 128)
    a = B.Attn(8, 1, 128, B.BF16, 16, case.num_blocks, case.max_blocks_per_seq, case.softmax_scale, 0, 0, 0)
    assert B.prefill_workspace_bytes(1, 48, 48, 9000, a) > 0
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    got = G.prefill_case(case, G.cache_for_case(case))
    _check(got, want, "bf16")


def test_generic_kernel_bf16_and_other_head_dims(oracle, G):
    for dtype, D, hq_l, hkv_l in [("bf16", 64, 4, 2), ("f32", 128, 8, 1), ("f32", 32, 2, 2), ("bf16", 256, 2, 1)]:
        case = W.make_attn_case("t", 54, dtype, [(37, 150), (80, 80), (1, 9)], hq_l, hkv_l, D)
        want = oracle.attention_case(case, oracle.cache_for_case(case))
        got = G.prefill_case(case, G.cache_for_case(case))
        _check(got, want, dtype)


DECODE_LENS = [1, 15, 16, 17, 31, 32, 33, 100, 511, 512, 513, 1023, 1500, 3000]


@pytest.mark.parametrize("hq_l,hkv_l", [(8, 1), (4, 1), (4, 4), (16, 1), (6, 2), (16, 2), (5, 1), (10, 2)])
def test_decode_bf16_small(oracle, G, hq_l, hkv_l):
    case = W.make_attn_case("t", 55, "bf16", [(1, c) for c in DECODE_LENS], hq_l, hkv_l, 128, pool_factor=1.3)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    got = G.decode_case(case, G.cache_for_case(case))
    _check(got, want, "bf16")


def test_decode_random_batches(oracle, G):
    """Thirty decode batches of random shape (1-40 sequences, contexts of 1-5000 tokens, 4 / 5 / 8 / 16 query heads per KV
    head), N(0,1) data: every output element within the bound (short contexts give single V rows of magnitude up to 4,
    where one bf16 step is 0.031)."""
    rng = np.random.default_rng(321)
    for it in range(30):
        n = int(rng.integers(1, 41))
        seqs = [(1, int(rng.integers(1, 5001)) if rng.integers(0, 4) else int(rng.integers(1, 40))) for _ in range(n)]
        hq = int(rng.choice([4, 5, 8, 16]))
        case = W.make_attn_case("dsweep", 2000 + it, "bf16", seqs, hq, 1, 128)
        want = oracle.attention_case(case, oracle.cache_for_case(case))
        got = W.to_f64(G.decode_case(case, G.cache_for_case(case)), "bf16")
        err = np.abs(got - want)
        assert err.max() <= 2e-2 and err.mean() <= 1e-3, (it, err.max(), err.mean())


def test_decode_many_sequences_and_long_contexts(oracle, G):
    """The flat decomposition at the edges of its range: as many (sequence, KV head) pairs as it
    indexes, one more than that (a second run of the kernel takes the rest), a context long enough that the
    minimum range per wavefront is set by the merge kernel's part limit, and a batch so small that
    most wavefronts get no tokens."""
    rng = np.random.default_rng(62)
    for n_seqs, hq_l, hkv_l in [(2048, 4, 1), (2049, 4, 1), (1024, 4, 2), (1025, 4, 2)]:
        lens = rng.integers(1, 70, size=n_seqs)
        case = W.make_attn_case("t", 63, "bf16", [(1, int(c)) for c in lens], hq_l, hkv_l, 128, pool_factor=1.2)
        want = oracle.attention_case(case, oracle.cache_for_case(case))
        _check(G.decode_case(case, G.cache_for_case(case)), want, "bf16")
    case = W.make_attn_case("t", 64, "bf16", [(1, 150001), (1, 3), (1, 40000)], 8, 1, 128, pool_factor=1.05)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    _check(G.decode_case(case, G.cache_for_case(case)), want, "bf16")
    case = W.make_attn_case("t", 65, "bf16", [(1, 2)], 8, 1, 128)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    _check(G.decode_case(case, G.cache_for_case(case)), want, "bf16")


def test_decode_fused_kv_write_and_fp32(oracle, G):
    from paper_2509_16495_amd import binding as B
    case = W.make_attn_case("t", 56, "bf16", [(1, c) for c in (1, 16, 17, 700, 64)], 8, 1, 128)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    cache = G.cache_for_case(case, only_cached=True)
    got = G.decode_case(case, cache, fused_new_kv=True)
    _check(got, want, "bf16")
    assert B.to_host(cache).tobytes() == oracle.cache_for_case(case).tobytes()
    case = W.make_attn_case("t", 57, "f32", [(1, c) for c in (1, 33, 200)], 4, 1, 64)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    _check(G.decode_case(case, G.cache_for_case(case)), want, "f32")


@pytest.mark.parametrize("dtype,D,fp8", [("bf16", 128, False), ("bf16", 128, True), ("f32", 64, False), ("bf16", 64, True)])
def test_decode_padding_rows_are_zero(oracle, G, dtype, D, fp8):
    """A batch padded to a fixed size (Sec. 3.4: the engine replays graphs captured per batch size): sequences of
    length 0 among the real ones, with a negative slot and a table row of invalid ids.  Their output rows are zero,
    every other row is what it is without them, and the cache is left as the real rows' appends make it."""
    import torch
    from paper_2509_16495_amd import binding as B
    case = W.make_attn_case("t", 66, dtype, [(1, c) for c in (40, 1, 333, 17, 64)], 4, 2, D, pool_factor=1.3)
    scales = (0.0371, 0.0293) if fp8 else None
    ref_cache = oracle.cache_for_case(case, fp8_scales=scales)
    want = oracle.attention_case(case, ref_cache, **(dict(k_scale=scales[0], v_scale=scales[1]) if fp8 else {}))
    pad_at = [0, 3, 7]                        # positions of the padding rows in the padded batch
    n = case.num_seqs + len(pad_at)
    real = [i for i in range(n) if i not in pad_at]
    lens = np.zeros(n, np.int32)
    lens[real] = case.ctx_lens
    table = np.full((n, case.block_table.shape[1]), -1, np.int32)
    table[real] = case.block_table
    slots = np.full(n, -1, np.int64)
    slots[real] = case.slots[case.new_token_index]
    q = np.zeros((n,) + case.q.shape[1:], case.q.dtype)
    q[real] = case.q
    k_new = np.zeros((n,) + case.k_ctx.shape[1:], case.k_ctx.dtype)
    v_new = np.zeros_like(k_new)
    k_new[real], v_new[real] = case.k_ctx[case.new_token_index], case.v_ctx[case.new_token_index]
    cache = G.cache_for_case(case, only_cached=True, fp8_scales=scales)
    out = torch.full((n, case.hq_l, D), 7.0, dtype=G.torch_dtype(dtype), device=G.DEV)
    kw = dict(k_scale=scales[0], v_scale=scales[1]) if fp8 else {}
    B.decode(G.t(q, dtype), cache, G.ti(table, np.int32), G.ti(lens, np.int32), int(lens.max()), out, case.softmax_scale,
             k_new=G.t(k_new, dtype), v_new=G.t(v_new, dtype), slot_mapping=G.ti(slots, np.int64), **kw)
    torch.cuda.synchronize()
    got = W.to_f64(B.to_host(out), dtype)
    assert np.all(got[pad_at] == 0.0)
    err = np.abs(got[real] - want)
    if dtype == "f32":
        assert err.max() <= F32_MAX, err.max()
    else:
        assert err.max() <= BF16_MAX and err.mean() <= BF16_MEAN, (err.max(), err.mean())
    assert B.to_host(cache).tobytes() == ref_cache.tobytes()
    # a batch of nothing but padding (max_seq_len 0): all rows zero, cache untouched
    out.fill_(7.0)
    lens[:] = 0
    slots[:] = -1
    B.decode(G.t(q, dtype), cache, G.ti(table, np.int32), G.ti(lens, np.int32), 0, out, case.softmax_scale,
             k_new=G.t(k_new, dtype), v_new=G.t(v_new, dtype), slot_mapping=G.ti(slots, np.int64), **kw)
    torch.cuda.synchronize()
    assert np.all(W.to_f64(B.to_host(out), dtype) == 0.0)
    assert B.to_host(cache).tobytes() == ref_cache.tobytes()


@pytest.mark.parametrize("hq,hkv", [(8, 1), (4, 2), (16, 1)])
def test_decode_appends_the_new_token_itself(oracle, G, hq, hkv):
    """Decode with the new tokens' K/V handed to the call (one launch writes and attends): contexts that end at
    every offset of a block and of a 32-token group."""
    from paper_2509_16495_amd import binding as B
    ctx = list(range(1, 70)) + [255, 256, 257, 1000, 1024, 4097]
    case = W.make_attn_case("dec_append", 83, "bf16", [(1, c) for c in ctx], hq, hkv, 128, pool_factor=1.4)
    ocache = oracle.cache_for_case(case)
    cache = G.cache_for_case(case, only_cached=True)
    got = G.decode_case(case, cache, fused_new_kv=True)
    assert B.to_host(cache).tobytes() == ocache.tobytes()
    _check(got, oracle.attention_case(case, ocache), "bf16")


def test_unwritten_cache_slots_may_hold_nan(oracle, G):
    """Slots past a sequence's context are never written; whatever they hold must not leak."""
    case = W.make_attn_case("t", 58, "bf16", [(1, 5), (1, 41), (1, 530)], 8, 1, 128)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    got = G.decode_case(case, G.cache_for_case(case, fill_byte=0xFF))       # 0xFFFF = bf16 NaN
    _check(got, want, "bf16")
    case = W.make_attn_case("t", 59, "bf16", [(37, 37), (5, 70)], 8, 1, 128)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    got = G.prefill_case(case, G.cache_for_case(case, fill_byte=0xFF))
    _check(got, want, "bf16")


def test_results_are_bitwise_reproducible(G):
    case = W.make_attn_case("t", 60, "bf16", [(1, c) for c in (900, 2100, 40)], 8, 1, 128)
    cache = G.cache_for_case(case)
    assert G.decode_case(case, cache).tobytes() == G.decode_case(case, cache).tobytes()
    case = W.make_attn_case("t", 61, "bf16", [(48, 9000), (200, 200)], 8, 1, 128)
    cache = G.cache_for_case(case)
    assert G.prefill_case(case, cache).tobytes() == G.prefill_case(case, cache).tobytes()


# ------------------------------------------------------------------------------------------------------
# benchmark-sized configurations, in the launch configuration the benchmark times
# ------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("data_scaled", [False, True])
def test_config2_8b_prefill_sampled(oracle, G, data_scaled):
    case = W.config2_attn(data_scaled=data_scaled)
    rows = _sample_rows(case, 24, 2)
    want = oracle.attention_case(case, oracle.cache_for_case(case), rows)
    got = G.prefill_case(case, G.cache_for_case(case))
    _check(got[rows], want, "bf16", relative=data_scaled)


def test_config3_70b_prefill_sampled(oracle, G):
    case = W.config3_attn()
    rows = _sample_rows(case, 40, 3)
    want = oracle.attention_case(case, oracle.cache_for_case(case), rows)
    got = G.prefill_case(case, G.cache_for_case(case))
    _check(got[rows], want, "bf16")


def test_config4_batch_decode_full(oracle, G):
    """Every output row of the 256-sequence batch; the cache (its 1.1 M context tokens written by the K/V write the
    benchmark times, the new tokens appended by the decode call) byte for byte."""
    from paper_2509_16495_amd import binding as B
    case = W.config4_attn()
    ocache = oracle.cache_for_case(case)
    want = oracle.attention_case(case, ocache)
    cache = G.cache_for_case(case, only_cached=True)
    got = G.decode_case(case, cache, fused_new_kv=True)
    _check(got, want, "bf16")
    assert B.to_host(cache).tobytes() == ocache.tobytes()


@pytest.mark.parametrize("dtype,D,hq,hkv", [("bf16", 128, 8, 1), ("bf16", 128, 4, 2), ("f32", 64, 4, 1)])
def test_mixed_batch_one_call(oracle, G, dtype, D, hq, hkv):
    """Chunks and decode rows in one call: same results and same cache as the oracle's write-then-attend, with either
    part empty as well."""
    from paper_2509_16495_amd import binding as B
    chunks = [(70, 70), (33, 200), (0, 5), (1, 1), (128, 300)]
    decodes = [(1, 1), (1, 17), (1, 250), (1, 64), (1, 1000), (1, 33)]
    for seqs, n_pre in ((chunks + decodes, len(chunks)), (chunks, len(chunks)), (decodes, 0)):
        case = W.make_attn_case("mixed_small", 77, dtype, seqs, hq, hkv, D, pool_factor=1.5)
        ocache = oracle.cache_for_case(case)
        cache = G.cache_for_case(case, only_cached=True)
        got = G.mixed_case(case, n_pre, cache)
        assert B.to_host(cache).tobytes() == ocache.tobytes()
        _check(got, oracle.attention_case(case, ocache), dtype)


def test_config5_mixed_step_one_call(oracle, G):
    """The long-context step through the unified entry point."""
    from paper_2509_16495_amd import binding as B
    case, n_prefill = W.config5_attn()
    ocache = oracle.cache_for_case(case)
    cache = G.cache_for_case(case, only_cached=True)
    got = G.mixed_case(case, n_prefill, cache)
    assert B.to_host(cache).tobytes() == ocache.tobytes()
    n_chunk = int(case.q_lens[:n_prefill].sum())
    # every 16th row of the chunk, all rows of its first and last column tile (32 tokens of 8 heads), every decode row
    chunk_rows = np.unique(np.concatenate([np.arange(0, n_chunk, 16), np.arange(0, 32), np.arange(n_chunk - 32, n_chunk)]))
    rows = np.concatenate([chunk_rows, np.arange(n_chunk, case.total_q)])
    _check(got[rows], oracle.attention_case(case, ocache, rows), "bf16")


def test_config5_mixed_step(oracle, G):
    """One 2048-token chunk on a 131072-token cached context plus 64 decodes in one block pool; the new
    tokens' K/V are written by the calls themselves."""
    from paper_2509_16495_amd import binding as B
    case, n_prefill = W.config5_attn()
    ocache = oracle.cache_for_case(case)
    cache = G.cache_for_case(case, only_cached=True)
    pre = W.sub_case(case, range(n_prefill))
    dec = W.sub_case(case, range(n_prefill, case.num_seqs))
    got_pre = G.prefill_case(pre, cache, fused_new_kv=True)
    got_dec = G.decode_case(dec, cache, fused_new_kv=True)
    assert B.to_host(cache).tobytes() == ocache.tobytes()
    rows = _sample_rows(pre, 8, 5, edge=8)
    _check(got_pre[rows], oracle.attention_case(pre, ocache, rows), "bf16")
    _check(got_dec, oracle.attention_case(dec, ocache), "bf16")
