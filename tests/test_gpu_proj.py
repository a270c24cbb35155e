"""GPU parity of the projections fused with the exchange layouts (Algorithm 1: qkv = embed * W_qkv written into the
send buffers; embed = unpack(recv) * W_o) against the CPU float64 oracle, through the C ABI.

Tolerance: bf16 operands are exact in both; the kernel accumulates K products in float32 (relative error of the
sum below K * 2^-24 of the sum of magnitudes) and rounds the result once to bf16 (relative 2^-9).  With N(0,1)
operands a result has magnitude ~sqrt(K), so: |err| <= 2^-8 |ref| + 1e-3 sqrt(K).  Padding rows must be exact zeros,
and every byte of the send buffers must be defined."""
import numpy as np
import pytest

from paper_2509_16495_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_backend
    return gpu_backend


def _bf16(rng, shape):
    return W.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


def _check(got_bits, want, K):
    got = W.to_f64(got_bits, "bf16")
    assert got.shape == want.shape and np.all(np.isfinite(got))
    err = np.abs(got - want)
    assert np.all(err <= 2.0 ** -8 * np.abs(want) + 1e-3 * np.sqrt(K)), float((err - 2.0 ** -8 * np.abs(want)).max())


QKV_CASES = [
    # P, h, h_kv, d_model, T, T_pad
    (8, 32, 8, 512, 300, 304),     # 8B-shaped heads; ragged tile, padding rows
    (8, 32, 4, 256, 70, 72),       # fewer KV heads than ranks: replication into several send buffers
    (4, 40, 8, 320, 257, 260),     # five query heads per KV head; d_model no multiple of 128
    (1, 2, 1, 64, 5, 5),           # one k step, one tile
    (2, 8, 4, 1024, 600, 600),     # three token tiles
    (8, 64, 8, 192, 0, 8),         # padding rows only
    (8, 64, 8, 128, 1800, 1800),   # 320 tiles: more than one per compute unit (the grid walks them), two k stages
]


@pytest.mark.parametrize("P,h,h_kv,d_model,T,T_pad", QKV_CASES)
def test_qkv_projection_into_send_buffers(oracle, G, P, h, h_kv, d_model, T, T_pad):
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(201))
    D = 128
    x, w = _bf16(rng, (T, d_model)), _bf16(rng, ((h + 2 * h_kv) * D, d_model))
    want = oracle.qkv_proj_pack(x, w, P, h, h_kv, D, T_pad, "bf16")
    send = torch.empty((P, T_pad, h // P + 2 * B.local_kv_heads(P, h_kv), D), dtype=torch.bfloat16, device=G.DEV)
    send.view(torch.uint8).fill_(0x55)
    B.qkv_proj_pack(G.t(x, "bf16"), G.t(w, "bf16"), send, P, h, h_kv)
    torch.cuda.synchronize()
    got = B.to_host(send)
    _check(got, want, d_model)
    assert not np.any(got[:, T:])          # padding rows: all-zero bits


@pytest.mark.parametrize("P,hq_l,d_model,T,T_pad", [(8, 4, 512, 300, 304), (4, 10, 256, 257, 260), (1, 2, 256, 5, 5),
                                                    (2, 4, 768, 600, 600), (8, 8, 256, 0, 4),
                                                    # eight tiles, one per XCD: every start of the k walk, most of them inside a source buffer's segment
                                                    (2, 3, 512, 1024, 1024)])
def test_o_projection_out_of_receive_buffers(oracle, G, P, hq_l, d_model, T, T_pad):
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(202))
    D = 128
    recv, w_o = _bf16(rng, (P, T_pad, hq_l, D)), _bf16(rng, (d_model, P * hq_l * D))
    want = oracle.unpack_o_proj(recv, w_o, T, "bf16")
    out = torch.empty((T, d_model), dtype=torch.bfloat16, device=G.DEV)
    out.view(torch.uint8).fill_(0x55)
    B.unpack_o_proj(G.t(recv, "bf16"), G.t(w_o, "bf16"), out)
    torch.cuda.synchronize()
    _check(B.to_host(out), want, P * hq_l * D)


def test_projection_then_attention_inputs_equal_separate_pack(oracle, G):
    """The fused projection leaves exactly the bytes that projecting into [T, heads, D] (rounded to bf16 the same
    way) and then packing would leave: checked by packing the kernel's own unfused result (P = 1 send buffer)."""
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(203))
    P, h, h_kv, D, d_model, T = 8, 32, 4, 128, 256, 200
    x, w = G.t(_bf16(rng, (T, d_model)), "bf16"), G.t(_bf16(rng, ((h + 2 * h_kv) * D, d_model)), "bf16")
    flat = torch.empty((1, T, h + 2 * h_kv, D), dtype=torch.bfloat16, device=G.DEV)
    B.qkv_proj_pack(x, w, flat, 1, h, h_kv)                       # P = 1: plain [T, heads, D]
    fused = torch.empty((P, T, h // P + 2, D), dtype=torch.bfloat16, device=G.DEV)
    B.qkv_proj_pack(x, w, fused, P, h, h_kv)
    packed = torch.empty_like(fused)
    B.pack_seq2head(flat[0], packed, P, h, h_kv)
    torch.cuda.synchronize()
    assert torch.equal(fused.view(torch.uint8), packed.view(torch.uint8))


def test_full_size_70b_projections_on_sampled_tokens(oracle, G):
    """The shapes the benchmark times (16384 tokens, d_model 8192, 64 + 2 x 8 heads, 8 buffers): every output of a
    sample of token rows (tile borders, first, last, random) against the oracle run on those rows alone."""
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(204))
    P, h, h_kv, D, d_model, T = 8, 64, 8, 128, 8192, 16384
    tokens = np.unique(np.concatenate([[0, 1, 127, 128, 255, 256, 257, 8191, 8192, 16127, 16128, 16383], rng.integers(0, T, 8)]))
    x, w = _bf16(rng, (T, d_model)), _bf16(rng, ((h + 2 * h_kv) * D, d_model))
    send = torch.empty((P, T, h // P + 2 * B.local_kv_heads(P, h_kv), D), dtype=torch.bfloat16, device=G.DEV)
    send.view(torch.uint8).fill_(0x55)
    B.qkv_proj_pack(G.t(x, "bf16"), G.t(w, "bf16"), send, P, h, h_kv)
    torch.cuda.synchronize()
    got = B.to_host(send[:, torch.from_numpy(tokens).to(G.DEV)].contiguous())
    want = oracle.qkv_proj_pack(x[tokens], w, P, h, h_kv, D, len(tokens), "bf16")
    _check(got, want, d_model)
    del send, x, w
    recv, w_o = _bf16(rng, (P, T, h // P, D)), _bf16(rng, (d_model, h * D))
    out = torch.empty((T, d_model), dtype=torch.bfloat16, device=G.DEV)
    out.view(torch.uint8).fill_(0x55)
    B.unpack_o_proj(G.t(recv, "bf16"), G.t(w_o, "bf16"), out)
    torch.cuda.synchronize()
    got = B.to_host(out[torch.from_numpy(tokens).to(G.DEV)].contiguous())
    want = oracle.unpack_o_proj(np.ascontiguousarray(recv[:, tokens]), w_o, len(tokens), "bf16")
    _check(got, want, h * D)
