"""One attention layer of an SP group, end to end through the C ABI, on one GPU (the ranks run one after the other,
the two all-to-alls are done by slicing, as in the oracle's virtual exchange): Algorithm 1 from the QKV projection
to the output projection.

    rank r:  send_r = qkv_proj_pack(embed_r)                 (projection written into the send buffers)
    a2a #1:  fused_r = rows of every rank's send_p[r]         (all tokens, head block r; KV heads replicated if needed)
    rank r:  attn_r = prefill(fused_r) with its K/V appended to rank r's cache
    a2a #2:  recv_r[p] = attn_p[tokens of rank r]
    rank r:  embed_r = unpack_o_proj(recv_r)

against the unsharded float64 computation (project, attend over all heads, project) whose intermediate q|k|v and
attention output are rounded to bf16 where the kernels round them.  This is a composition check, not a parity gate:
every kernel has its own element-wise test; here the rounding of two intermediates may fall differently in a few
elements, so the comparison is on the relative RMS error and a generous element bound."""
import numpy as np
import pytest

from paper_2509_16495_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_backend
    return gpu_backend


def _round_bf16(a64):
    return W.to_f64(W.f32_to_bf16_bits(a64.astype(np.float32)), "bf16")


@pytest.mark.parametrize("P,h,h_kv", [(2, 8, 2), (4, 8, 2)])     # (4, 8, 2): fewer KV heads than ranks, replication
def test_sp_layer_slice_matches_unsharded_float64(oracle, G, P, h, h_kv):
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(401))
    D, d_model = 128, 256
    geo = W.make_attn_case("slice", 402, "bf16", [(150, 150), (41, 41), (65, 65)], 1, 1, D, pool_factor=1.5)   # block tables / slots only
    n = geo.total_q                                   # 256 tokens, all new (prefill from empty caches)
    assert n % P == 0
    T = n // P
    hq_l, hkv_l = h // P, max(1, h_kv // P)
    x = W.f32_to_bf16_bits(rng.standard_normal((n, d_model), dtype=np.float32))
    w_qkv = W.f32_to_bf16_bits(rng.standard_normal(((h + 2 * h_kv) * D, d_model), dtype=np.float32) * np.float32(d_model ** -0.5))
    w_o = W.f32_to_bf16_bits(rng.standard_normal((d_model, h * D), dtype=np.float32) * np.float32((h * D) ** -0.5))
    xd, wq, wo = G.t(x, "bf16"), G.t(w_qkv, "bf16"), G.t(w_o, "bf16")

    # ---- GPU, rank by rank ----
    sends = []
    for r in range(P):
        send = torch.empty((P, T, hq_l + 2 * hkv_l, D), dtype=torch.bfloat16, device=G.DEV)
        B.qkv_proj_pack(xd[r * T:(r + 1) * T].contiguous(), wq, send, P, h, h_kv)
        sends.append(send)
    table, cu, lens = G.ti(geo.block_table, np.int32), G.ti(geo.cu_seqlens_q, np.int32), G.ti(geo.ctx_lens, np.int32)
    slots = G.ti(geo.slots, np.int64)
    attn = []
    for r in range(P):
        fused = torch.cat([sends[p][r] for p in range(P)], dim=0)                      # first all-to-all
        cache = G.new_cache(geo.num_blocks, hkv_l, D, "bf16")
        out = torch.empty((n, hq_l, D), dtype=torch.bfloat16, device=G.DEV)
        B.prefill(fused[:, :hq_l], cache, table, cu, lens, int(geo.q_lens.max()), int(geo.ctx_lens.max()), out, geo.softmax_scale,
                  k_new=fused[:, hq_l:hq_l + hkv_l], v_new=fused[:, hq_l + hkv_l:], slot_mapping=slots)
        attn.append(out)
    embed = []
    for r in range(P):
        recv = torch.stack([attn[p][r * T:(r + 1) * T] for p in range(P)], dim=0).contiguous()   # second all-to-all
        e = torch.empty((T, d_model), dtype=torch.bfloat16, device=G.DEV)
        B.unpack_o_proj(recv, wo, e)
        embed.append(e)
    torch.cuda.synchronize()
    got = W.to_f64(B.to_host(torch.cat(embed, dim=0)), "bf16")

    # ---- unsharded float64 ----
    qkv = _round_bf16(W.to_f64(x, "bf16") @ W.to_f64(w_qkv, "bf16").T).reshape(n, h + 2 * h_kv, D)
    q, k, v = qkv[:, :h], qkv[:, h:h + h_kv], qkv[:, h + h_kv:]
    a = np.zeros((n, h, D))
    for s in range(geo.num_seqs):
        lo, hi = int(geo.cu_seqlens_q[s]), int(geo.cu_seqlens_q[s + 1])
        a[lo:hi] = oracle.attention_dense_np(q[lo:hi], k[lo:hi], v[lo:hi], geo.softmax_scale, hi - lo)
    want = _round_bf16(a).reshape(n, h * D) @ W.to_f64(w_o, "bf16").T
    err = got - want
    rel_rms = np.sqrt(np.mean(err ** 2) / np.mean(want ** 2))
    assert rel_rms < 1e-2, rel_rms
    assert np.all(np.abs(err) <= 2.0 ** -6 * np.abs(want) + 0.05 * np.sqrt(np.mean(want ** 2))), float(np.abs(err).max())
