"""Both tuned prefill kernels (128-column and 256-column workgroup tiles) against the fp64 oracle, each forced
through shiftattn_set_option so that no shape escapes either of them, with and without forced key splits.

Tolerances as for all bf16 attention: max |err| <= 2e-2 and mean |err| <= 1e-3 against the oracle.
"""
import numpy as np
import pytest

from paper_2509_16495_amd import workloads as W

pytestmark = pytest.mark.gpu

BF16_MAX, BF16_MEAN = 2e-2, 1e-3


@pytest.fixture(scope="module")
def G():
    import gpu_backend
    return gpu_backend


@pytest.fixture
def opts():
    """Sets tuning switches for one test and puts them back to 'decided per call'."""
    from paper_2509_16495_amd import binding as B

    def set_(tile=0, splits=0, pairing=0, scaled_q=0):
        B.set_option(B.OPT_PREFILL_TILE, tile)
        B.set_option(B.OPT_PREFILL_SPLITS, splits)
        B.set_option(B.OPT_PREFILL_PAIRING, pairing)
        B.set_option(B.OPT_PREFILL_SCALED_Q, scaled_q)

    yield set_
    B.set_option(B.OPT_PREFILL_TILE, 0)
    B.set_option(B.OPT_PREFILL_SPLITS, 0)
    B.set_option(B.OPT_PREFILL_PAIRING, 0)
    B.set_option(B.OPT_PREFILL_SCALED_Q, 0)


def _check(got_bits, want):
    got = W.to_f64(got_bits, "bf16")
    assert got.shape == want.shape
    assert np.all(np.isfinite(got))
    err = np.abs(got - want)
    assert err.max() <= BF16_MAX and err.mean() <= BF16_MEAN, (err.max(), err.mean())


SHAPES = [
    # seqs (q_len, ctx), hq_l, hkv_l
    ([(200, 200), (77, 300), (1, 50), (130, 130)], 8, 1),   # several tiles, ragged tails, chunked, a one-token chunk
    ([(64, 64), (33, 33), (16, 16)], 4, 1),
    ([(150, 150), (5, 260)], 8, 2),                          # two KV heads
    ([(100, 100)], 4, 4),                                    # no GQA sharing: 256 tokens per wide tile
    ([(90, 190)], 6, 2),                                     # three query heads per KV head
    ([(300, 300)], 16, 1),
    ([(0, 10), (40, 40), (0, 0)], 4, 1),                     # empty chunks in the batch
    ([(140, 140), (31, 333)], 5, 1),                         # 40q/8kv model on 8 ranks (Table 4): 51 tokens per wide tile
    ([(129, 200)], 10, 2),
    ([(700, 700)], 8, 1),                                    # 22 wide tiles: pairs, a middle tile on its own
    ([(513, 1100), (31, 31), (257, 257)], 8, 1),             # several sequences of unequal tile counts
    ([(40, 4000)], 7, 1),                                    # 36 tokens per wide tile, long cached context
    # short chunks behind long contexts (longest context >= 16 x longest chunk): the wide kernel takes one tile per
    # workgroup instead of pairs; sequences of 4, 1, 3 and 0 tiles, one of them a prefill from nothing
    ([(100, 2100), (31, 31), (70, 1200), (0, 5)], 8, 1),
    ([(65, 1100), (64, 1040)], 8, 2),
]


@pytest.mark.parametrize("tile", [128, 256])
@pytest.mark.parametrize("splits", [0, 3])
@pytest.mark.parametrize("seqs,hq_l,hkv_l", SHAPES)
def test_prefill_kernel_forced(oracle, G, opts, tile, splits, seqs, hq_l, hkv_l):
    from paper_2509_16495_amd import binding as B
    opts(tile=tile, splits=splits)
    assert B.get_option(B.OPT_PREFILL_TILE) == tile and B.get_option(B.OPT_PREFILL_SPLITS) == splits
    case = W.make_attn_case("t", 91, "bf16", seqs, hq_l, hkv_l, 128)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    got = G.prefill_case(case, G.cache_for_case(case, fill_byte=0xFF))   # unwritten slots hold NaN patterns
    _check(got, want)


@pytest.mark.parametrize("pairing", [1, 2])
@pytest.mark.parametrize("splits", [0, 2])
@pytest.mark.parametrize("seqs,hq_l,hkv_l", SHAPES)
def test_wide_prefill_kernel_tiles_in_pairs_and_one_per_workgroup(oracle, G, opts, pairing, splits, seqs, hq_l, hkv_l):
    """The 256-column kernel with its tiles forced two per workgroup (heaviest with lightest) and one per workgroup
    (heaviest first), whatever the planner would choose for the shape."""
    opts(tile=256, splits=splits, pairing=pairing)
    case = W.make_attn_case("t", 93, "bf16", seqs, hq_l, hkv_l, 128)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    got = G.prefill_case(case, G.cache_for_case(case, fill_byte=0xFF))
    _check(got, want)


@pytest.mark.parametrize("splits", [0, 3])
@pytest.mark.parametrize("seqs,hq_l,hkv_l", SHAPES)
def test_wide_prefill_kernel_on_scaled_q(oracle, G, opts, splits, seqs, hq_l, hkv_l):
    """The 256-column kernel with SHIFTATTN_OPT_PREFILL_SCALED_Q (off by default): Q takes the softmax scale when a tile
    fetches it and is rounded to bf16 again, which moves a logit by up to 2^-9 of its value.  An output may then land one
    bf16 step (at most 2^-7 of its magnitude) from the correctly rounded value, so the bound on the largest error is the
    usual one plus that step; the bound on the mean error is the usual one."""
    opts(tile=256, splits=splits, scaled_q=1)
    case = W.make_attn_case("t", 95, "bf16", seqs, hq_l, hkv_l, 128)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    got = W.to_f64(G.prefill_case(case, G.cache_for_case(case, fill_byte=0xFF)), "bf16")
    assert got.shape == want.shape and np.all(np.isfinite(got))
    err = np.abs(got - want)
    assert np.all(err <= BF16_MAX + 2.0 ** -7 * np.abs(want)) and err.mean() <= BF16_MEAN, (err.max(), err.mean())


@pytest.mark.parametrize("tile", [128, 256])
def test_prefill_fused_append_and_fp8_cache_forced(oracle, G, opts, tile):
    from paper_2509_16495_amd import binding as B
    opts(tile=tile)
    case = W.make_attn_case("t", 92, "bf16", [(70, 170), (128, 128), (1, 40), (300, 900)], 8, 1, 128)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    cache = G.cache_for_case(case, only_cached=True)
    _check(G.prefill_case(case, cache, fused_new_kv=True), want)
    assert B.to_host(cache).tobytes() == oracle.cache_for_case(case).tobytes()
    scales = (0.0371, 0.0293)
    ocache = oracle.cache_for_case(case, fp8_scales=scales)
    want = oracle.attention_case(case, ocache, k_scale=scales[0], v_scale=scales[1])
    cache = G.cache_for_case(case, only_cached=True, fp8_scales=scales)
    _check(G.prefill_case(case, cache, fused_new_kv=True, fp8_scales=scales), want)
    assert B.to_host(cache).tobytes() == ocache.tobytes()


def _with_late_outliers(case, rows, key_positions, beta):
    """Copies of the case's K in which, for each listed (query row, key position) pair of sequence 0, the key is beta
    times that row's query vector of head 0: that logit exceeds everything before it by tens of nats."""
    q = W.bf16_bits_to_f32(case.q)
    k = W.bf16_bits_to_f32(case.k_ctx).copy()
    for row, pos in zip(rows, key_positions):
        k[pos, 0] = beta * q[row, 0]
    case.k_ctx = W.f32_to_bf16_bits(k)
    return case


@pytest.mark.parametrize("tile,beta", [(128, 3.0), (256, 3.0), (256, 9.0)])
def test_prefill_reference_maximum_jumps_late(oracle, G, opts, tile, beta):
    """Logits that exceed a column's running maximum by far more than the kernels let their reference lag, long after the
    column has begun to accumulate: the 128-column kernel rescales in place, the 256-column kernel runs the pass again
    from the final reference.  Also a jump inside the very first key tile and one in the last, partial tile.  beta = 3:
    about 50 powers of two above everything before (the 256-column kernel's first attempt, which follows no maximum behind
    the first tile, still holds it); beta = 9: about 150 (its running sums leave the fp32 range it allows itself, the
    pass is run again following the maximum, and once more from the final reference)."""
    opts(tile=tile)
    case = W.make_attn_case("t", 93, "bf16", [(300, 1500)], 8, 1, 128)
    first_new = 1200
    rows = [5, 5, 120, 299, 17]
    keys = [700, 1100, 3, first_new + 299, 40]       # visible to their rows: key <= 1200 + row
    case = _with_late_outliers(case, rows, keys, beta=beta)
    want = oracle.attention_case(case, oracle.cache_for_case(case))
    got = G.prefill_case(case, G.cache_for_case(case))
    _check(got, want)
    # the affected rows are dominated by one key: their result is that key's V row to within the tolerance
    v = W.to_f64(case.v_ctx, "bf16")
    g = W.to_f64(got, "bf16")
    assert np.abs(g[299, 0] - v[first_new + 299, 0]).max() <= BF16_MAX


@pytest.mark.parametrize("tile", [128, 256])
def test_prefill_random_batches(oracle, G, opts, tile):
    """Forty batches of random shape (1-4 sequences, chunks of 1-700 tokens, a third of them behind up to 3000 cached
    tokens, 4 / 5 / 8 / 16 query heads per KV head), N(0,1) data: every output element within the bound.  The first rows of
    a prompt are single V rows of magnitude up to 4, where one bf16 step is 0.031: the bound of 2e-2 holds there only if
    the largest probability of such a row is exact (a softmax without a reference failed two of these forty)."""
    opts(tile=tile)
    rng = np.random.default_rng(123)
    for it in range(40):
        seqs = []
        for _ in range(int(rng.integers(1, 5))):
            q = int(rng.integers(1, 700))
            seqs.append((q, q + int(rng.integers(0, 3) == 0) * int(rng.integers(0, 3000))))
        hq = int(rng.choice([4, 5, 8, 16]))
        case = W.make_attn_case("sweep", 1000 + it, "bf16", seqs, hq, 1, 128)
        want = oracle.attention_case(case, oracle.cache_for_case(case))
        got = G.prefill_case(case, G.cache_for_case(case))
        _check(got, want)


def test_prefill_kernels_agree_on_dispatch(oracle, G, opts):
    """Left to itself the library picks a kernel per launch; whichever it picks, results stay within tolerance of the
    oracle on a shape at the boundary of the choice (enough 256-column tiles to fill the chip, or not)."""
    for n_tok in (1500, 6300):
        case = W.make_attn_case("t", 94, "bf16", [(n_tok, n_tok)], 8, 1, 128)
        rows = np.unique(np.concatenate([np.arange(0, 40), np.arange(n_tok - 40, n_tok),
                                         np.random.default_rng(4).integers(0, n_tok, 24)]))
        want = oracle.attention_case(case, oracle.cache_for_case(case), rows)
        got = G.prefill_case(case, G.cache_for_case(case))
        _check(got[rows], want)
