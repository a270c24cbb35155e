"""Pins for the CPU oracle's FP8 E4M3 KV cache (no GPU).

The format is pinned to the published OCP 8-bit floating point definition (E4M3: bias 7, no infinities,
S.1111.111 = NaN, largest finite 448, smallest subnormal 2^-9) through its constants, through torch's CPU
float8_e4m3fn type (an independent implementation of the same format) and through the rounding rule's own
properties.  The write is pinned by plain numpy indexing of the cache arrangement, the attention by the
unquantised oracle run over the values the codes stand for.  The paper (Sec. 4.1) only says that an FP8 KV
cache was used; format and scale rule are this build's convention.
"""
import numpy as np
import pytest
import torch

from paper_2509_16495_amd import workloads as W

FINITE = [c for c in range(256) if (c & 0x7F) != 0x7F]


def test_format_constants(oracle):
    v = oracle.e4m3_value
    assert v(0x7E) == 448.0 and v(0xFE) == -448.0          # largest finite: 1.75 * 2^8
    assert v(0x38) == 1.0 and v(0x40) == 2.0 and v(0x3C) == 1.5
    assert v(0x08) == 2.0 ** -6                            # smallest normal
    assert v(0x01) == 2.0 ** -9 and v(0x07) == 7 * 2.0 ** -9  # subnormals: m * 2^-9
    assert v(0x00) == 0.0 and v(0x80) == 0.0 and np.signbit(v(0x80))
    assert np.isnan(v(0x7F)) and np.isnan(v(0xFF))
    vals = [v(c) for c in range(0x7F)]
    assert all(b > a for a, b in zip(vals, vals[1:]))      # codes ascend with their values


def test_values_match_torch_float8(oracle):
    want = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = np.array([oracle.e4m3_value(c) for c in range(256)])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    fin = ~np.isnan(want)
    assert np.array_equal(got[fin], want[fin]) and np.array_equal(np.signbit(got[fin]), np.signbit(want[fin]))


def test_encode_round_trip_ties_and_saturation(oracle):
    enc, val = oracle.e4m3_from_float, oracle.e4m3_value
    for c in FINITE:
        assert enc(val(c)) == c, hex(c)
    for c in range(0x7E):                                   # midpoint of neighbours goes to the even code
        mid = 0.5 * (val(c) + val(c + 1))
        assert enc(mid) == (c if c % 2 == 0 else c + 1), hex(c)
        assert enc(-mid) == 0x80 | (c if c % 2 == 0 else c + 1)
        just_below, just_above = np.nextafter(np.float32(mid), np.float32(0)), np.nextafter(np.float32(mid), np.float32(1e9))
        assert enc(float(just_below)) == c and enc(float(just_above)) == c + 1
    for big in (448.0, 449.0, 464.0, 480.0, 1e6, 3e38, float("inf")):
        assert enc(big) == 0x7E and enc(-big) == 0xFE       # saturating, never NaN
    assert enc(float("nan")) & 0x7F == 0x7F
    assert enc(2.0 ** -10) == 0x00 and enc(np.nextafter(np.float32(2.0 ** -10), np.float32(1))) == 0x01  # tie at half the smallest step
    assert enc(1e-30) == 0x00 and enc(-1e-30) == 0x80


def test_encode_matches_torch_in_range(oracle):
    rng = np.random.Generator(np.random.PCG64(8))
    x = np.concatenate([rng.standard_normal(4000) * s for s in (1e-3, 0.02, 1.0, 30.0, 150.0)]).astype(np.float32)
    x = x[np.abs(x) <= 448.0]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_from_float(float(v)) for v in x], dtype=np.uint8)
    assert np.array_equal(got, want)


def test_rounding_error_bound(oracle):
    rng = np.random.Generator(np.random.PCG64(9))
    for x in (rng.standard_normal(2000) * 20).astype(np.float32):
        c = oracle.e4m3_from_float(float(x))
        a = abs(float(x))
        step = 2.0 ** -9 if a < 2.0 ** -6 else 2.0 ** (np.floor(np.log2(a)) - 3)   # spacing of the binade of x
        assert abs(oracle.e4m3_value(c) - float(x)) <= 0.5 * step * (1 + 1e-7)


def _torch_codes(x_f64, scale):
    y = (x_f64.astype(np.float32) / np.float32(scale)).astype(np.float32)
    y = np.clip(y, -448.0, 448.0)
    return torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_write_places_codes_like_plain_indexing(oracle, dtype):
    case = W.make_attn_case("w8", 21, dtype, [(5, 37), (1, 16), (9, 9)], 4, 2, 16, pool_factor=1.5)
    ks, vs = 0.0625, 0.03125
    cache = oracle.cache_for_case(case, fp8_scales=(ks, vs))
    B, D, hkv = case.block_size, case.D, case.hkv_l
    want = np.full_like(cache, 0xA5)
    kc, vc = _torch_codes(W.to_f64(case.k_ctx, dtype), ks), _torch_codes(W.to_f64(case.v_ctx, dtype), vs)
    for i, slot in enumerate(case.slots):
        blk, off = divmod(int(slot), B)
        for g in range(hkv):
            want[blk, g, 0].reshape(B, D)[off] = kc[i, g]          # K: token-major
            want[blk, g, 1].reshape(D, B)[:, off] = vc[i, g]       # V: dimension-major
    assert np.array_equal(cache, want)
    # padding rows (negative slots) write nothing
    slots = case.slots.copy()
    slots[::2] = -1
    c2 = oracle.new_cache(case.num_blocks, hkv, B, D, "fp8_e4m3")
    oracle.kv_write_fp8(c2, case.k_ctx, case.v_ctx, slots, B, dtype, ks, vs)
    c3 = oracle.new_cache(case.num_blocks, hkv, B, D, "fp8_e4m3")
    oracle.kv_write_fp8(c3, case.k_ctx[1::2], case.v_ctx[1::2], case.slots[1::2], B, dtype, ks, vs)
    assert np.array_equal(c2, c3)


def test_write_quotient_is_taken_in_float32(oracle):
    """x / scale with a scale that is no power of two: the code is that of the float32 quotient."""
    rng = np.random.Generator(np.random.PCG64(10))
    k = (rng.standard_normal((64, 1, 16)) * 3).astype(np.float32)
    scale = np.float32(0.0123)
    cache = oracle.new_cache(4, 1, 16, 16, "fp8_e4m3")
    oracle.kv_write_fp8(cache, k, k, np.arange(64), 16, "f32", float(scale), float(scale))
    want = _torch_codes(k.astype(np.float64), scale)
    assert np.array_equal(cache[:, 0, 0].reshape(64, 16), want[:, 0])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention_over_codes_equals_attention_over_their_values(oracle, dtype):
    case = W.make_attn_case("a8", 22, dtype, [(6, 40), (1, 23), (17, 17)], 4, 2, 16, pool_factor=1.5)
    ks, vs = 0.0625, 0.125   # powers of two: code value * scale is exact in float32
    c8 = oracle.cache_for_case(case, fp8_scales=(ks, vs))
    got = oracle.attention_case(case, c8, k_scale=ks, v_scale=vs)
    deq = np.zeros(c8.shape, dtype=np.float32)
    table = np.array([oracle.e4m3_value(c) for c in range(256)])
    deq[:, :, 0] = table[c8[:, :, 0]] * ks   # unwritten slots hold the sentinel byte, a finite code; never read
    deq[:, :, 1] = table[c8[:, :, 1]] * vs
    qf = W.to_f64(case.q, dtype).astype(np.float32)
    want = oracle.attention(qf, deq, "f32", case.block_table, case.cu_seqlens_q, case.ctx_lens, case.hq_l, case.hkv_l,
                            case.D, case.block_size, case.softmax_scale)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    # and stays close to the unquantised result: E4M3 keeps 4 significant bits
    exact = oracle.attention_case(case, oracle.cache_for_case(case))
    assert np.abs(got - exact).max() < 0.25 and np.abs(got - exact).mean() < 0.03


def test_scales_fold_into_softmax_scale_and_output(oracle):
    case = W.make_attn_case("s8", 23, "bf16", [(4, 30), (1, 50)], 2, 1, 16)
    c8 = oracle.cache_for_case(case, fp8_scales=(0.05, 0.02))
    a = oracle.attention_case(case, c8, k_scale=0.05, v_scale=0.02)
    b = oracle.attention(case.q, c8, "bf16", case.block_table, case.cu_seqlens_q, case.ctx_lens, case.hq_l, case.hkv_l,
                         case.D, case.block_size, case.softmax_scale * 0.05, None, "fp8_e4m3", 1.0, 1.0) * 0.02
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-15)
