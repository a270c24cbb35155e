"""Decode steps of few sequences (the regime of the shift configuration, Algorithm 2) against the fp64 oracle: one to
64 sequences, contexts from one token to tens of thousands, so that a row has anything from one part to several
hundred.  max |err| <= 2e-2 and mean |err| <= 1e-3 for bf16; the parts of a row are merged in a fixed order, so the
output is bitwise reproducible as well."""
import numpy as np
import pytest
import torch

from paper_2509_16495_amd import workloads as W

pytestmark = pytest.mark.gpu

BF16_MAX, BF16_MEAN = 2e-2, 1e-3


@pytest.fixture(scope="module")
def G():
    import gpu_backend
    return gpu_backend


def _check(got_bits, want):
    got = W.to_f64(got_bits, "bf16")
    assert np.all(np.isfinite(got))
    err = np.abs(got - want)
    assert err.max() <= BF16_MAX and err.mean() <= BF16_MEAN, (err.max(), err.mean())


BATCHES = [
    # context lengths, hq_l, hkv_l
    ([4097], 8, 1),
    ([4097] * 4, 8, 1),
    ([1, 15, 16, 17, 31, 32, 33, 100, 511, 512, 513, 1023, 1500, 3000], 8, 1),
    ([40000], 8, 1),                                  # several hundred parts for each row
    ([33000, 5, 64, 9000], 4, 2),                     # two KV heads per sequence
    ([700] * 64, 8, 1),
    ([3000, 2, 800] * 7, 16, 1),
    ([257, 64, 1000], 5, 1),
]


@pytest.mark.parametrize("ctx,hq_l,hkv_l", BATCHES)
def test_small_decode_batches(oracle, G, ctx, hq_l, hkv_l):
    from paper_2509_16495_amd import binding as B
    case = W.make_attn_case("t", 95, "bf16", [(1, c) for c in ctx], hq_l, hkv_l, 128, pool_factor=1.3)
    ocache = oracle.cache_for_case(case)
    want = oracle.attention_case(case, ocache)
    cache = G.cache_for_case(case, only_cached=True, fill_byte=0xFF)
    got = G.decode_case(case, cache, fused_new_kv=True)
    _check(got, want)
    # appended K/V bytes: compare the written slots only (the rest of the pool holds the fill pattern on one side)
    assert B.to_host(G.cache_for_case(case)).tobytes() == ocache.tobytes()
    assert G.decode_case(case, cache).tobytes() == G.decode_case(case, cache).tobytes()


def test_small_decode_batch_fp8_cache_and_padding_rows(oracle, G):
    from paper_2509_16495_amd import binding as B
    scales = (0.0371, 0.0293)
    case = W.make_attn_case("t", 96, "bf16", [(1, c) for c in (40, 1, 5000, 17, 640)], 8, 1, 128, pool_factor=1.3)
    ref_cache = oracle.cache_for_case(case, fp8_scales=scales)
    want = oracle.attention_case(case, ref_cache, k_scale=scales[0], v_scale=scales[1])
    cache = G.cache_for_case(case, only_cached=True, fp8_scales=scales)
    _check(G.decode_case(case, cache, fused_new_kv=True, fp8_scales=scales), want)
    assert B.to_host(cache).tobytes() == ref_cache.tobytes()
    # padding rows (length 0) among real ones: zero output rows, nothing appended for them
    pad_at = [0, 3]
    n = case.num_seqs + len(pad_at)
    real = [i for i in range(n) if i not in pad_at]
    lens = np.zeros(n, np.int32)
    lens[real] = case.ctx_lens
    table = np.full((n, case.block_table.shape[1]), -1, np.int32)
    table[real] = case.block_table
    q = np.zeros((n,) + case.q.shape[1:], case.q.dtype)
    q[real] = case.q
    out = torch.full((n, case.hq_l, 128), 7.0, dtype=torch.bfloat16, device=G.DEV)
    B.decode(G.t(q, "bf16"), cache, G.ti(table, np.int32), G.ti(lens, np.int32), int(lens.max()), out, case.softmax_scale,
             k_scale=scales[0], v_scale=scales[1])
    torch.cuda.synchronize()
    got = W.to_f64(B.to_host(out), "bf16")
    assert np.all(got[pad_at] == 0.0)
    err = np.abs(got[real] - want)
    assert err.max() <= BF16_MAX and err.mean() <= BF16_MEAN
