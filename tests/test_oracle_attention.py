"""Pins for the CPU oracle's attention (no GPU).

The oracle is checked against things other than itself: brute force with an
explicit probability matrix, closed forms, torch's CPU float64 attention, and
the invariances the method relies on (head shards concatenate to unsharded
attention; chunked prefill and decode are rows of a full prefill; block-table
permutations do not change a bit; split-K partials merge exactly).
"""
import math

import numpy as np
import pytest

from paper_2509_16495_amd import workloads as W


def _dense(case, s=0):
    """float64 q [q_len,hq,D], k,v [ctx,hkv,D] of sequence s."""
    q = W.to_f64(case.q[case.cu_seqlens_q[s]:case.cu_seqlens_q[s + 1]], case.dtype)
    k = W.to_f64(case.k_ctx[case.cu_ctx[s]:case.cu_ctx[s + 1]], case.dtype)
    v = W.to_f64(case.v_ctx[case.cu_ctx[s]:case.cu_ctx[s + 1]], case.dtype)
    return q, k, v


def _run(oracle, case, rows=None):
    return oracle.attention_case(case, oracle.cache_for_case(case), rows)


def _brute_force(q, k, v, scale, q_len):
    """No max-subtraction, explicit [q_len x ctx] probability matrix, exact summation (fsum)."""
    ctx, hkv, D = k.shape
    hq = q.shape[1]
    out = np.zeros((q_len, hq, D))
    rowsum = np.zeros((q_len, hq))
    for i in range(q_len):
        pos = ctx - q_len + i
        for j in range(hq):
            g = j // (hq // hkv)
            w = [math.exp(scale * math.fsum(float(q[i, j, d]) * float(k[t, g, d]) for d in range(D)))
                 for t in range(pos + 1)]
            z = math.fsum(w)
            p = [x / z for x in w]
            rowsum[i, j] = math.fsum(p)
            for d in range(D):
                out[i, j, d] = math.fsum(p[t] * float(v[t, g, d]) for t in range(pos + 1))
    return out, rowsum


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_brute_force_tiny(oracle, dtype):
    case = W.make_attn_case("t", 11, dtype, [(7, 7), (3, 9), (1, 5)], 4, 2, 8)
    got = _run(oracle, case)
    for s in range(case.num_seqs):
        q, k, v = _dense(case, s)
        want, rowsum = _brute_force(q, k, v, case.softmax_scale, int(case.q_lens[s]))
        assert np.all(np.abs(rowsum - 1.0) <= 1e-12)
        np.testing.assert_allclose(got[case.cu_seqlens_q[s]:case.cu_seqlens_q[s + 1]], want, rtol=0, atol=1e-13)


def test_rows_sum_to_one_via_constant_v(oracle):
    case = W.make_attn_case("t", 12, "f32", [(40, 40), (5, 70)], 4, 1, 16)
    case.v_ctx[...] = 1.0
    got = _run(oracle, case)
    assert np.max(np.abs(got - 1.0)) <= 1e-12


def test_closed_forms(oracle):
    # ctx = 1 -> V[0]; first causal row -> V[0]
    case = W.make_attn_case("t", 13, "f32", [(1, 1), (6, 6)], 2, 1, 16)
    got = _run(oracle, case)
    _, _, v0 = _dense(case, 0)
    _, _, v1 = _dense(case, 1)
    for j in range(2):
        assert np.array_equal(got[0, j], v0[0, 0])
        assert np.array_equal(got[1, j], v1[0, 0])
    # all keys equal -> uniform weights -> running mean of V
    case = W.make_attn_case("t", 14, "f32", [(9, 9)], 2, 1, 16)
    case.k_ctx[...] = case.k_ctx[0:1]
    got = _run(oracle, case)
    _, _, v = _dense(case)
    for i in range(9):
        np.testing.assert_allclose(got[i, 0], v[: i + 1, 0].mean(axis=0), rtol=0, atol=1e-14)
    # one key aligned with q and huge -> output collapses to that key's V
    case = W.make_attn_case("t", 15, "f32", [(1, 12)], 1, 1, 16)
    case.k_ctx[...] *= 0.01
    case.k_ctx[5, 0] = case.q[0, 0] * 1000.0
    got = _run(oracle, case)
    np.testing.assert_allclose(got[0, 0], _dense(case)[2][5, 0], rtol=0, atol=1e-12)


def test_logit_shift_invariance(oracle):
    """Adding one vector u to every key shifts all logits of a query by q.u and changes nothing."""
    case = W.make_attn_case("t", 16, "f32", [(8, 20)], 2, 2, 8)
    a = _run(oracle, case)
    u = np.arange(8, dtype=np.float32) / 4  # exactly representable
    case.k_ctx[...] = (case.k_ctx.astype(np.float64) + u).astype(np.float32)
    b = _run(oracle, case)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-5)  # keys were re-rounded to fp32
    # exact version: scale keys' first coordinate only through q=0 there
    case = W.make_attn_case("t", 17, "f32", [(8, 20)], 2, 2, 8)
    case.q[:, :, 0] = 0.0
    a = _run(oracle, case)
    case.k_ctx[:, :, 0] += 7.0
    b = _run(oracle, case)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-15)


def test_against_torch_sdpa_float64(oracle):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    # full causal prefill -> is_causal=True
    case = W.make_attn_case("t", 18, "bf16", [(33, 33)], 4, 4, 32)
    got = _run(oracle, case)
    q, k, v = (torch.from_numpy(x).permute(1, 0, 2)[None] for x in _dense(case))
    want = F.scaled_dot_product_attention(q, k, v, is_causal=True, scale=case.softmax_scale)[0].permute(1, 0, 2)
    np.testing.assert_allclose(got, want.numpy(), rtol=0, atol=1e-12)
    # chunked prefill + GQA -> explicit bottom-right mask, KV heads expanded by repeat_interleave
    case = W.make_attn_case("t", 19, "bf16", [(10, 45)], 6, 2, 32)
    got = _run(oracle, case)
    q, k, v = (torch.from_numpy(x).permute(1, 0, 2)[None] for x in _dense(case))
    k, v = k.repeat_interleave(3, dim=1), v.repeat_interleave(3, dim=1)
    mask = torch.arange(45)[None, :] <= (35 + torch.arange(10))[:, None]
    want = F.scaled_dot_product_attention(q, k, v, attn_mask=mask, scale=case.softmax_scale)[0].permute(1, 0, 2)
    np.testing.assert_allclose(got, want.numpy(), rtol=0, atol=1e-12)


def test_against_numpy_statement(oracle):
    case = W.make_attn_case("t", 20, "f32", [(17, 50), (64, 64), (1, 100)], 8, 2, 64)
    got = _run(oracle, case)
    for s in range(case.num_seqs):
        q, k, v = _dense(case, s)
        want = oracle.attention_dense_np(q, k, v, case.softmax_scale, int(case.q_lens[s]))
        np.testing.assert_allclose(got[case.cu_seqlens_q[s]:case.cu_seqlens_q[s + 1]], want, rtol=0, atol=1e-12)


def test_head_shards_concatenate_to_unsharded(oracle):
    """Each of P ranks runs attention on its own head block; stacking the blocks in block order
    gives the attention of all heads (heads are independent: Sec. 2.3 'Head Parallelism')."""
    P, H, Hkv, D = 4, 8, 4, 16
    full = W.make_attn_case("t", 21, "bf16", [(12, 30), (20, 20)], H, Hkv, D)
    whole = _run(oracle, full)
    hq_l, hkv_l = H // P, Hkv // P
    for p in range(P):
        shard = W.make_attn_case("t", 21, "bf16", [(12, 30), (20, 20)], H, Hkv, D)
        shard.hq_l, shard.hkv_l = hq_l, hkv_l
        shard.q = np.ascontiguousarray(full.q[:, p * hq_l:(p + 1) * hq_l])
        shard.k_ctx = np.ascontiguousarray(full.k_ctx[:, p * hkv_l:(p + 1) * hkv_l])
        shard.v_ctx = np.ascontiguousarray(full.v_ctx[:, p * hkv_l:(p + 1) * hkv_l])
        part = _run(oracle, shard)
        assert np.array_equal(part, whole[:, p * hq_l:(p + 1) * hq_l])


def test_chunked_prefill_and_decode_are_rows_of_full_prefill(oracle):
    full = W.make_attn_case("t", 22, "f32", [(48, 48)], 4, 1, 16)
    whole = _run(oracle, full)
    for q_len in (1, 5, 16, 47):
        part = W.make_attn_case("t", 22, "f32", [(48, 48)], 4, 1, 16)
        part.q = np.ascontiguousarray(full.q[48 - q_len:])
        part.q_lens = np.array([q_len], dtype=np.int32)
        part.cu_seqlens_q = np.array([0, q_len], dtype=np.int32)
        got = oracle.attention_case(part, oracle.cache_for_case(full))
        np.testing.assert_allclose(got, whole[48 - q_len:], rtol=0, atol=1e-14)


def test_block_table_permutation_is_bit_invariant(oracle):
    kw = dict(seed=23, dtype="bf16", seqs=[(20, 77), (1, 33)], hq_l=4, hkv_l=2, D=16)
    a = W.make_attn_case("t", permute_blocks=False, pool_factor=1.0, **kw)
    b = W.make_attn_case("t", permute_blocks=True, pool_factor=3.0, **kw)
    assert np.array_equal(a.q, b.q) and np.array_equal(a.k_ctx, b.k_ctx)
    assert not np.array_equal(a.block_table, b.block_table)
    assert np.array_equal(_run(oracle, a), _run(oracle, b))


def test_row_subset_matches_full(oracle):
    case = W.make_attn_case("t", 24, "bf16", [(30, 30), (9, 40), (1, 17)], 4, 1, 16)
    whole = _run(oracle, case)
    rows = np.array([39, 0, 29, 30, 38, 7], dtype=np.int64)
    assert np.array_equal(_run(oracle, case, rows), whole[rows])


def test_splitk_merge_identity(oracle):
    rng = np.random.default_rng(25)
    k, v, q = rng.standard_normal((300, 32)), rng.standard_normal((300, 32)), rng.standard_normal(32)
    scale = 0.3
    one = oracle.splitk_combine(oracle.splitk_partials(q, k, v, scale, [0, 300]))
    s = scale * (k @ q)
    p = np.exp(s - s.max())
    np.testing.assert_allclose(one, (p / p.sum()) @ v, rtol=0, atol=1e-14)
    for bounds in ([0, 1, 300], [0, 64, 128, 192, 256, 300], [0, 299, 300], list(range(0, 301, 20))):
        many = oracle.splitk_combine(oracle.splitk_partials(q, k, v, scale, bounds))
        np.testing.assert_allclose(many, one, rtol=0, atol=1e-12)


def test_planted_mistakes_are_caught(oracle):
    """The pins above must fail for plausible slips; emulate three of them on the numpy statement
    (transposed GQA map, off-by-one mask, missing scale) and check the C oracle disagrees."""
    case = W.make_attn_case("t", 26, "f32", [(6, 9)], 4, 2, 8)
    got = _run(oracle, case)
    q, k, v = _dense(case)
    good = oracle.attention_dense_np(q, k, v, case.softmax_scale, 6)
    assert np.max(np.abs(got - good)) < 1e-12
    wrong_gqa = oracle.attention_dense_np(q[:, [0, 2, 1, 3]], k, v, case.softmax_scale, 6)[:, [0, 2, 1, 3]]
    off_by_one = oracle.attention_dense_np(q, k[:-1], v[:-1], case.softmax_scale, 6)
    no_scale = oracle.attention_dense_np(q, k, v, 1.0, 6)
    for bad in (wrong_gqa, off_by_one, no_scale):
        assert np.max(np.abs(got - bad)) > 1e-3


def test_empty_and_degenerate(oracle):
    case = W.make_attn_case("t", 27, "f32", [(0, 5), (3, 3), (0, 0)], 2, 1, 8)
    got = _run(oracle, case)
    assert got.shape == (3, 2, 8)
    none = W.make_attn_case("t", 28, "f32", [], 2, 1, 8)
    assert _run(oracle, none).shape == (0, 2, 8)
