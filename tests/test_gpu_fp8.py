"""GPU parity of the FP8 E4M3 KV cache against the CPU oracle, through the C ABI.

The cache bytes must be identical to the oracle's (the code of an element is decided by a float32
quotient and a nearest-even rounding on both sides); attention over such a cache is compared with the
oracle's attention over the same codes, to the bf16 / fp32 tolerances of the unquantised path - the
quantisation error itself is common to both sides and not part of the comparison.
"""
import numpy as np
import pytest

from paper_2509_16495_amd import workloads as W

pytestmark = pytest.mark.gpu

BF16_MAX, BF16_MEAN, F32_MAX = 2e-2, 1e-3, 1e-5
SCALES = (0.0371, 0.0293)   # no powers of two: the quotient rounds


@pytest.fixture(scope="module")
def G():
    import gpu_backend
    return gpu_backend


def _check(got_bits, want, dtype):
    got = W.to_f64(got_bits, dtype)
    assert got.shape == want.shape and np.all(np.isfinite(got))
    err = np.abs(got - want)
    if dtype == "f32":
        assert err.max() <= F32_MAX, err.max()
    else:
        assert err.max() <= BF16_MAX and err.mean() <= BF16_MEAN, (err.max(), err.mean())


@pytest.mark.parametrize("dtype,D,hkv", [("bf16", 128, 1), ("bf16", 64, 2), ("f32", 64, 1), ("f32", 128, 3)])
def test_quantising_write_is_bit_exact(oracle, G, dtype, D, hkv):
    """Codes over five decades of magnitude, values that saturate, ragged and skipped slots."""
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(31))
    n, nb = 777, 64
    mag = 10.0 ** rng.uniform(-4.5, 1.5, size=(n, hkv, D))
    k = (rng.standard_normal((n, hkv, D)) * mag).astype(np.float32)
    v = (rng.standard_normal((n, hkv, D)) * mag[::-1]).astype(np.float32)
    k[5, 0, :8] = [0.0, -0.0, 1e-30, -1e-30, 1e30, -1e30, 448 * SCALES[0], 464 * SCALES[0]]
    if dtype == "bf16":
        k, v = W.f32_to_bf16_bits(k), W.f32_to_bf16_bits(v)
    slots = rng.permutation(nb * 16)[:n].astype(np.int64)
    slots[rng.integers(0, n, size=40)] = -1
    want = oracle.new_cache(nb, hkv, 16, D, "fp8_e4m3")
    oracle.kv_write_fp8(want, k, v, slots, 16, dtype, *SCALES)
    cache = G.new_cache_fp8(nb, hkv, D)
    G.kv_write(cache, k, v, slots, dtype, SCALES)
    got = B.to_host(cache)
    assert got.dtype == np.uint8 and got.tobytes() == want.tobytes()


@pytest.mark.parametrize("dtype,D,hq,hkv", [("bf16", 128, 8, 1), ("bf16", 128, 4, 2), ("bf16", 64, 4, 1), ("f32", 64, 4, 2)])
def test_prefill_decode_and_mixed_over_fp8_cache(oracle, G, dtype, D, hq, hkv):
    from paper_2509_16495_amd import binding as B
    chunks = [(70, 70), (33, 200), (0, 5), (1, 1), (128, 300)]
    decodes = [(1, 1), (1, 17), (1, 250), (1, 64), (1, 1000), (1, 33)]
    case = W.make_attn_case("mixed_fp8", 78, dtype, chunks + decodes, hq, hkv, D, pool_factor=1.5)
    n_pre = len(chunks)
    ocache = oracle.cache_for_case(case, fp8_scales=SCALES)
    want = oracle.attention_case(case, ocache, k_scale=SCALES[0], v_scale=SCALES[1])
    n_chunk = int(case.q_lens[:n_pre].sum())
    # one unified call that also writes the new tokens
    cache = G.cache_for_case(case, only_cached=True, fp8_scales=SCALES)
    got = G.mixed_case(case, n_pre, cache, fp8_scales=SCALES)
    assert B.to_host(cache).tobytes() == ocache.tobytes()
    _check(got, want, dtype)
    # the two kinds of rows through their own entry points over the finished cache
    pre, dec = W.sub_case(case, range(n_pre)), W.sub_case(case, range(n_pre, case.num_seqs))
    _check(G.prefill_case(pre, cache, fp8_scales=SCALES), want[:n_chunk], dtype)
    _check(G.decode_case(dec, cache, fp8_scales=SCALES), want[n_chunk:], dtype)


def test_decode_fp8_many_sequences_long_contexts(oracle, G):
    """Decode batch that spans many wavefront ranges: 96 sequences, contexts 1..6000, 8q/1kv."""
    rng = np.random.Generator(np.random.PCG64(32))
    ctx = np.concatenate([[1, 15, 16, 17, 31, 32, 33, 6000], rng.integers(1, 4000, size=88)])
    case = W.make_attn_case("dec_fp8", 79, "bf16", [(1, int(c)) for c in ctx], 8, 1, 128, pool_factor=1.2)
    ocache = oracle.cache_for_case(case, fp8_scales=SCALES)
    cache = G.cache_for_case(case, fp8_scales=SCALES)
    got = G.decode_case(case, cache, fp8_scales=SCALES)
    _check(got, oracle.attention_case(case, ocache, k_scale=SCALES[0], v_scale=SCALES[1]), "bf16")


def test_chunked_prefill_fp8_long_context_with_key_splits(oracle, G):
    """A short chunk on a long cached context (keys split over workgroups, partials merged) next to ordinary
    prefills, all over an FP8 cache that the call widens into its workspace."""
    case = W.make_attn_case("chunk_fp8", 80, "bf16", [(96, 9000), (300, 300), (40, 1234)], 8, 1, 128, pool_factor=1.3)
    ocache = oracle.cache_for_case(case, fp8_scales=SCALES)
    cache = G.cache_for_case(case, only_cached=True, fp8_scales=SCALES)
    got = G.prefill_case(case, cache, fused_new_kv=True, fp8_scales=SCALES)
    from paper_2509_16495_amd import binding as B
    assert B.to_host(cache).tobytes() == ocache.tobytes()
    _check(got, oracle.attention_case(case, ocache, k_scale=SCALES[0], v_scale=SCALES[1]), "bf16")


def test_decode_fp8_more_pairs_than_the_flat_kernel_indexes(oracle, G):
    """2100 (sequence, KV head) pairs: more than one launch of the decode kernel indexes, served in two runs."""
    rng = np.random.Generator(np.random.PCG64(33))
    ctx = rng.integers(1, 120, size=2100)
    case = W.make_attn_case("dec_fp8_many", 81, "bf16", [(1, int(c)) for c in ctx], 8, 1, 128, pool_factor=1.1)
    ocache = oracle.cache_for_case(case, fp8_scales=SCALES)
    cache = G.cache_for_case(case, fp8_scales=SCALES)
    got = G.decode_case(case, cache, fp8_scales=SCALES)
    _check(got, oracle.attention_case(case, ocache, k_scale=SCALES[0], v_scale=SCALES[1]), "bf16")


@pytest.mark.parametrize("hq,hkv", [(8, 1), (4, 2)])
def test_decode_fp8_appends_the_new_token_itself(oracle, G, hq, hkv):
    """Decode with the new tokens' K/V handed to the call: the cache ends up with the oracle's codes and the new
    token is attended to (contexts that end at every offset of a block and of a 32-token group)."""
    from paper_2509_16495_amd import binding as B
    ctx = list(range(1, 70)) + [255, 256, 257, 1000, 1024, 4097]
    case = W.make_attn_case("dec_fp8_append", 82, "bf16", [(1, c) for c in ctx], hq, hkv, 128, pool_factor=1.4)
    ocache = oracle.cache_for_case(case, fp8_scales=SCALES)
    cache = G.cache_for_case(case, only_cached=True, fp8_scales=SCALES)
    got = G.decode_case(case, cache, fused_new_kv=True, fp8_scales=SCALES)
    assert B.to_host(cache).tobytes() == ocache.tobytes()
    _check(got, oracle.attention_case(case, ocache, k_scale=SCALES[0], v_scale=SCALES[1]), "bf16")


# ------------------------------------------------------------------------------------------------------
# benchmark-sized configurations over an FP8 cache, in the launch configuration the benchmark times.  The oracle's
# quantiser is a linear search per element, so it writes the contexts of sampled sequences only (into a cache of
# the full pool's shape); the GPU runs the whole batch.
# ------------------------------------------------------------------------------------------------------
def _blocks_of(case, seq_ids):
    return np.concatenate([case.block_table[s, :(int(case.ctx_lens[s]) + 15) // 16] for s in seq_ids])


def test_config4_batch_decode_fp8_sampled_sequences(oracle, G):
    """256 decode sequences, contexts U[512, 8192], over an FP8 cache; the new tokens are quantised and appended by
    the call.  The shortest, the longest and four random sequences: output rows against the oracle, their cache
    blocks byte for byte."""
    from paper_2509_16495_amd import binding as B
    case = W.config4_attn()
    rng = np.random.default_rng(4)
    ids = sorted({int(np.argmin(case.ctx_lens)), int(np.argmax(case.ctx_lens)), *map(int, rng.integers(0, case.num_seqs, size=4))})
    sub = W.sub_case(case, ids)
    ocache = oracle.cache_for_case(sub, fp8_scales=SCALES)
    cache = G.cache_for_case(case, only_cached=True, fp8_scales=SCALES)
    got = G.decode_case(case, cache, fused_new_kv=True, fp8_scales=SCALES)
    blocks = _blocks_of(case, ids)
    assert B.to_host(cache)[blocks].tobytes() == ocache[blocks].tobytes()
    _check(got[ids], oracle.attention_case(sub, ocache, k_scale=SCALES[0], v_scale=SCALES[1]), "bf16")


def test_config5_mixed_step_fp8_one_call_sampled(oracle, G):
    """The long-context step (2048-token chunk on 131072 cached tokens + 64 decodes) over an FP8 cache through the
    unified entry point.  The chunk's sequence and two decode sequences: their cache blocks byte for byte, sampled
    chunk rows and the two decode rows against the oracle."""
    from paper_2509_16495_amd import binding as B
    case, n_prefill = W.config5_attn()
    assert n_prefill == 1
    dec_lens = case.ctx_lens[n_prefill:]
    ids = [0, n_prefill + int(np.argmin(dec_lens)), n_prefill + int(np.argsort(dec_lens)[len(dec_lens) // 2])]
    sub = W.sub_case(case, ids)
    ocache = oracle.cache_for_case(sub, fp8_scales=SCALES)
    cache = G.cache_for_case(case, only_cached=True, fp8_scales=SCALES)
    got = G.mixed_case(case, n_prefill, cache, fp8_scales=SCALES)
    blocks = _blocks_of(case, ids)
    assert B.to_host(cache)[blocks].tobytes() == ocache[blocks].tobytes()
    n_chunk = int(case.q_lens[0])
    rng = np.random.default_rng(5)
    chunk_rows = np.unique(np.concatenate([np.arange(8), np.arange(n_chunk - 8, n_chunk), rng.integers(0, n_chunk, size=8)]))
    rows_sub = np.concatenate([chunk_rows, [n_chunk, n_chunk + 1]])                     # rows of the sub-case
    rows_all = np.concatenate([chunk_rows, [n_chunk + i - n_prefill for i in ids[1:]]])   # the same rows of the batch
    want = oracle.attention_case(sub, ocache, rows_sub, k_scale=SCALES[0], v_scale=SCALES[1])
    _check(got[rows_all], want, "bf16")
