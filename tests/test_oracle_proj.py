"""Pins for the oracle's projections next to the exchange (no GPU): Algorithm 1's qkv = embed * W_qkv in front of
the first all-to-all and embed = attn_o * W_o behind the second.  The matrix product is numpy's float64 matmul,
pinned here by an explicit triple loop with exact summation; the layouts are pinned by the byte-moving pack /
unpack of the same oracle and by identity weights."""
import math

import numpy as np
import pytest
import torch

from paper_2509_16495_amd import workloads as W


def _rand(rng, shape, dtype):
    x = rng.standard_normal(shape).astype(np.float32)
    return W.f32_to_bf16_bits(x) if dtype == "bf16" else x


@pytest.mark.parametrize("dtype,P,h,h_kv", [("bf16", 2, 4, 2), ("f32", 4, 4, 1), ("bf16", 1, 2, 0)])
def test_qkv_projection_against_explicit_loops(oracle, dtype, P, h, h_kv):
    rng = np.random.Generator(np.random.PCG64(101))
    T, T_pad, d, D = 5, 6, 7, 4
    x, w = _rand(rng, (T, d), dtype), _rand(rng, ((h + 2 * h_kv) * D, d), dtype)
    got = oracle.qkv_proj_pack(x, w, P, h, h_kv, D, T_pad, dtype)
    x64, w64 = W.to_f64(x, dtype), W.to_f64(w, dtype)
    y = np.array([[math.fsum(float(x64[t, k]) * float(w64[n, k]) for k in range(d)) for n in range(w.shape[0])] for t in range(T)])
    want = oracle.pack_heads_f64(y.reshape(T, h + 2 * h_kv, D), P, h, h_kv, T_pad)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    assert np.all(got[:, T:] == 0.0)


@pytest.mark.parametrize("P,h,h_kv", [(8, 32, 4), (4, 40, 8), (2, 8, 4), (3, 6, 6)])
def test_pack_of_float64_rows_moves_what_the_byte_pack_moves(oracle, P, h, h_kv):
    rng = np.random.Generator(np.random.PCG64(102))
    T, T_pad, D = 9, 11, 8
    y = rng.standard_normal((T, h + 2 * h_kv, D)).astype(np.float32)
    a = oracle.pack_heads_f64(y.astype(np.float64), P, h, h_kv, T_pad)
    b = oracle.pack_seq2head(y, P, h, h_kv, T_pad, "f32")
    assert np.array_equal(a.astype(np.float32), b)


def test_identity_weights_reduce_the_projections_to_pack_and_unpack(oracle):
    rng = np.random.Generator(np.random.PCG64(103))
    P, h, h_kv, D, T, T_pad = 2, 4, 2, 4, 6, 6
    n = (h + 2 * h_kv) * D
    x = _rand(rng, (T, n), "bf16")
    eye = W.f32_to_bf16_bits(np.eye(n, dtype=np.float32))
    got = oracle.qkv_proj_pack(x, eye, P, h, h_kv, D, T_pad, "bf16")
    want = oracle.pack_seq2head(x.reshape(T, h + 2 * h_kv, D), P, h, h_kv, T_pad, "bf16")
    assert np.array_equal(got, W.to_f64(want, "bf16"))
    recv = _rand(rng, (P, T_pad, h // P, D), "bf16")
    eye_o = W.f32_to_bf16_bits(np.eye(h * D, dtype=np.float32))
    got_o = oracle.unpack_o_proj(recv, eye_o, T, "bf16")
    want_o = oracle.unpack_head2seq(recv, T, "bf16").reshape(T, h * D)
    assert np.array_equal(got_o, W.to_f64(want_o, "bf16"))


def test_o_projection_against_explicit_loops(oracle):
    rng = np.random.Generator(np.random.PCG64(104))
    P, hq_l, D, T, T_pad, d = 3, 2, 4, 5, 7, 6
    recv, w_o = _rand(rng, (P, T_pad, hq_l, D), "bf16"), _rand(rng, (d, P * hq_l * D), "bf16")
    got = oracle.unpack_o_proj(recv, w_o, T, "bf16")
    r64, w64 = W.to_f64(recv, "bf16"), W.to_f64(w_o, "bf16")
    want = np.zeros((T, d))
    for t in range(T):
        for c in range(d):
            want[t, c] = math.fsum(float(r64[p, t, j, e]) * float(w64[c, (p * hq_l + j) * D + e])
                                   for p in range(P) for j in range(hq_l) for e in range(D))
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


# ---- FP8 E4M3 operands with per-row scales ------------------------------------------------------------------------
def _torch_row_quant(x64):
    """Independent restatement with torch's CPU float8 type: amax / 448 and x / scale in float32."""
    x = torch.from_numpy(x64.astype(np.float32))
    amax = x.abs().amax(dim=1)
    scale = torch.where(amax > 0, amax / np.float32(448.0), torch.ones_like(amax))
    q = (x / scale[:, None]).clamp(-448.0, 448.0)
    return q.to(torch.float8_e4m3fn).view(torch.uint8).numpy(), scale.numpy()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_row_quantisation_against_torch_float8(oracle, dtype):
    rng = np.random.Generator(np.random.PCG64(110))
    x = _rand(rng, (37, 96), dtype)
    x64 = W.to_f64(x, dtype).copy()
    x64[5] = 0.0                                         # a zero row keeps scale 1 and all-zero codes
    x64[6] *= 1e-3
    x64[7] *= 300.0
    x = W.f32_to_bf16_bits(x64.astype(np.float32)) if dtype == "bf16" else x64.astype(np.float32)
    x64 = W.to_f64(x, dtype)
    codes, scales = oracle.quantize_rows_e4m3(x, dtype)
    want_codes, want_scales = _torch_row_quant(x64)
    assert np.array_equal(scales, want_scales) and scales[5] == 1.0 and not codes[5].any()
    assert np.array_equal(codes, want_codes)
    # the element of largest magnitude of every non-zero row becomes +-448, nothing saturates beyond it
    tab = oracle.e4m3_table()
    assert np.all(np.abs(tab[codes]).max(axis=1)[np.arange(37) != 5] == 448.0)
    # dequantised rows are within half an E4M3 step (2^-4 relative, or half the smallest subnormal step) of the input
    deq = tab[codes] * scales.astype(np.float64)[:, None]
    assert np.all(np.abs(deq - x64) <= 2.0 ** -4 * np.abs(x64) + 2.0 ** -10 * scales[:, None] + 1e-30)


def test_fp8_projections_against_explicit_loops(oracle):
    rng = np.random.Generator(np.random.PCG64(111))
    P, h, h_kv, D, T, T_pad, d = 2, 4, 2, 4, 5, 6, 9
    xc, xs = oracle.quantize_rows_e4m3(_rand(rng, (T, d), "bf16"), "bf16")
    wc, ws = oracle.quantize_rows_e4m3(_rand(rng, ((h + 2 * h_kv) * D, d), "bf16"), "bf16")
    got = oracle.qkv_proj_pack_fp8(xc, xs, wc, ws, P, h, h_kv, D, T_pad)
    val = oracle.e4m3_value
    y = np.array([[float(xs[t]) * float(ws[n]) * math.fsum(val(xc[t, k]) * val(wc[n, k]) for k in range(d))
                   for n in range(wc.shape[0])] for t in range(T)])
    want = oracle.pack_heads_f64(y.reshape(T, h + 2 * h_kv, D), P, h, h_kv, T_pad)
    np.testing.assert_allclose(got, want, rtol=1e-14, atol=0)
    # output projection: token rows gathered from the receive buffers
    hq_l, d_out = 2, 7
    rc, rs = oracle.quantize_rows_e4m3(_rand(rng, (T, P * hq_l * D), "bf16"), "bf16")
    recv_codes = np.zeros((P, T_pad, hq_l, D), dtype=np.uint8)
    for p in range(P):
        recv_codes[p, :T] = rc[:, p * hq_l * D:(p + 1) * hq_l * D].reshape(T, hq_l, D)
    assert np.array_equal(oracle.recv_rows(recv_codes, T), rc)
    woc, wos = oracle.quantize_rows_e4m3(_rand(rng, (d_out, P * hq_l * D), "bf16"), "bf16")
    got_o = oracle.unpack_o_proj_fp8(recv_codes, rs, woc, wos, T)
    want_o = np.array([[float(rs[t]) * float(wos[n]) * math.fsum(val(rc[t, k]) * val(woc[n, k]) for k in range(rc.shape[1]))
                        for n in range(d_out)] for t in range(T)])
    np.testing.assert_allclose(got_o, want_o, rtol=1e-14, atol=0)


def test_fp8_projection_of_exactly_representable_operands_equals_the_unquantised_one(oracle):
    """Small integers times a power of two are E4M3 values: quantising them loses nothing, so the FP8 projection
    must reproduce the bf16 projection of the same numbers exactly."""
    rng = np.random.Generator(np.random.PCG64(112))
    P, h, h_kv, D, T, d = 2, 4, 2, 4, 6, 16
    xi = rng.integers(-7, 8, size=(T, d)).astype(np.float32)
    xi[:, 0] = 7.0                                       # amax 7 in every row: scale 7 / 448 = 2^-6
    wi = rng.integers(-7, 8, size=((h + 2 * h_kv) * D, d)).astype(np.float32)
    wi[:, 1] = -7.0
    x, w = W.f32_to_bf16_bits(xi * 0.5), W.f32_to_bf16_bits(wi * 4.0)
    xc, xs = oracle.quantize_rows_e4m3(x, "bf16")
    wc, ws = oracle.quantize_rows_e4m3(w, "bf16")
    got = oracle.qkv_proj_pack_fp8(xc, xs, wc, ws, P, h, h_kv, D, T)
    want = oracle.qkv_proj_pack(x, w, P, h, h_kv, D, T, "bf16")
    assert np.array_equal(got, want)
