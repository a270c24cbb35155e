"""Pins for the oracle's projections next to the exchange (no GPU): Algorithm 1's qkv = embed * W_qkv in front of
the first all-to-all and embed = attn_o * W_o behind the second.  The matrix product is numpy's float64 matmul,
pinned here by an explicit triple loop with exact summation; the layouts are pinned by the byte-moving pack /
unpack of the same oracle and by identity weights."""
import math

import numpy as np
import pytest

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
