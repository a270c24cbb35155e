"""The projections for the few token rows of a decode step (Algorithm 2: the side of the threshold where batches are
small; Algorithm 1: the QKV and O products) against the CPU float64 oracle, through the C ABI: 1 to 64 rows take the
weight-streaming kernel (from 17 rows on with a workspace for its k groups), a few hundred rows the large-batch kernel
with k split over workgroups, and calls without a workspace the large-batch kernel as it is.  Tolerance as for all bf16 projections: |err| <= 2^-8 |ref| + 1e-3 sqrt(K); padding rows
are exact zeros, every byte of the outputs is written, and a call repeated gives the same bits."""
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


def _workspace(B, G, rows, n_features, k, give):
    import torch
    need = B.proj_workspace_bytes(rows, n_features, k)
    if not give:
        return None, need
    return torch.empty(max(need, 16), dtype=torch.uint8, device=G.DEV), need


QKV_SMALL = [
    # P, h, h_kv, d_model, T, T_pad
    (8, 64, 8, 8192, 1, 1),        # the 70B shard: one token
    (8, 64, 8, 8192, 8, 8),
    (8, 64, 8, 8192, 13, 16),      # padding rows
    (8, 64, 8, 8192, 17, 24),      # two token blocks, two k groups
    (8, 64, 8, 8192, 64, 64),      # four token blocks, four k groups
    (8, 32, 8, 4096, 8, 8),        # 8B-shaped: 24 features per workgroup, a ragged second tile
    (8, 32, 8, 4096, 40, 40),
    (8, 32, 4, 2048, 30, 32),      # fewer KV heads than ranks: replication into several send buffers
    (4, 40, 8, 1024, 5, 8),        # five query heads per KV head; 28 features per workgroup
    (1, 2, 1, 1024, 3, 3),         # fewer features than workgroups x 4
    (8, 64, 8, 5120, 8, 8),        # k not served by the streaming kernel: the large-batch kernel takes it
    (8, 64, 8, 8192, 100, 104),    # above 64 rows: the large-batch kernel, k split over six workgroups per tile
    (8, 64, 8, 8192, 256, 256),
    (8, 32, 8, 4096, 300, 304),    # two token tiles, five k ranges
    (2, 8, 4, 1024, 600, 600),     # short k: two ranges
]


@pytest.mark.parametrize("give_workspace", [True, False])
@pytest.mark.parametrize("P,h,h_kv,d_model,T,T_pad", QKV_SMALL)
def test_small_qkv_projection(oracle, G, P, h, h_kv, d_model, T, T_pad, give_workspace):
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(211))
    D = 128
    x, w = _bf16(rng, (T, d_model)), _bf16(rng, ((h + 2 * h_kv) * D, d_model))
    want = oracle.qkv_proj_pack(x, w, P, h, h_kv, D, T_pad, "bf16")
    ws, _ = _workspace(B, G, T_pad, (h + 2 * h_kv) * D, d_model, give_workspace)
    xd, wd = G.t(x, "bf16"), G.t(w, "bf16")
    runs = []
    for _ in range(2):
        send = torch.empty((P, T_pad, h // P + 2 * B.local_kv_heads(P, h_kv), D), dtype=torch.bfloat16, device=G.DEV)
        send.view(torch.uint8).fill_(0x55)
        B.qkv_proj_pack(xd, wd, send, P, h, h_kv, workspace=ws)
        torch.cuda.synchronize()
        runs.append(B.to_host(send))
    _check(runs[0], want, d_model)
    assert not np.any(runs[0][:, T:])
    assert runs[0].tobytes() == runs[1].tobytes()


O_SMALL = [
    # P, hq_l, d_model, T, T_pad
    (8, 8, 8192, 1, 1),
    (8, 8, 8192, 16, 16),
    (8, 8, 8192, 33, 40),
    (8, 8, 8192, 64, 64),
    (8, 4, 4096, 8, 8),
    (4, 10, 1024, 7, 8),           # k = 5120: not served by the streaming kernel
    (2, 4, 768, 20, 20),
    (1, 8, 256, 3, 4),
    (8, 8, 8192, 256, 256),        # the large-batch kernel with k split over five workgroups per tile
    (8, 4, 4096, 130, 136),
    (2, 4, 768, 300, 300),         # a k range that starts inside the second receive buffer
]


@pytest.mark.parametrize("give_workspace", [True, False])
@pytest.mark.parametrize("P,hq_l,d_model,T,T_pad", O_SMALL)
def test_small_o_projection(oracle, G, P, hq_l, d_model, T, T_pad, give_workspace):
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(212))
    D = 128
    recv, w_o = _bf16(rng, (P, T_pad, hq_l, D)), _bf16(rng, (d_model, P * hq_l * D))
    want = oracle.unpack_o_proj(recv, w_o, T, "bf16")
    ws, _ = _workspace(B, G, T, d_model, P * hq_l * D, give_workspace)
    rd, wd = G.t(recv, "bf16"), G.t(w_o, "bf16")
    runs = []
    for _ in range(2):
        out = torch.empty((T, d_model), dtype=torch.bfloat16, device=G.DEV)
        out.view(torch.uint8).fill_(0x55)
        B.unpack_o_proj(rd, wd, out, workspace=ws)
        torch.cuda.synchronize()
        runs.append(B.to_host(out))
    _check(runs[0], want, P * hq_l * D)
    assert runs[0].tobytes() == runs[1].tobytes()


def test_projection_workspace_sizes_and_a_short_workspace():
    """What the size query promises: nothing for up to 16 rows at k = 8192, k groups x token rows x features x 4 bytes
    above, nothing where the streaming kernel does not serve; a workspace shorter than that is not used (the call
    falls back to the kernel that needs none) rather than overrun."""
    import torch
    from paper_2509_16495_amd import binding as B
    assert B.proj_workspace_bytes(16, 10240, 8192) == 0
    assert B.proj_workspace_bytes(17, 10240, 8192) == 2 * 32 * 10240 * 4
    assert B.proj_workspace_bytes(64, 10240, 8192) == 4 * 64 * 10240 * 4
    assert B.proj_workspace_bytes(65, 10240, 8192) == 6 * 65 * 10240 * 4       # 40 output tiles: six k ranges each
    assert B.proj_workspace_bytes(256, 8192, 8192) == 6 * 256 * 8192 * 4
    assert B.proj_workspace_bytes(2048, 10240, 8192) == 3 * 512 * 10240 * 4    # 320 tiles: 240 whole, the last 512 rows in three k ranges
    assert B.proj_workspace_bytes(2048, 8192, 8192) == 0                       # 256 tiles: one round of the chip
    assert B.proj_workspace_bytes(16384, 10240, 8192) == 0                     # enough tiles without a split
    assert B.proj_workspace_bytes(64, 6144, 4096) == 2 * 64 * 6144 * 4
    assert B.proj_workspace_bytes(8, 10240, 5120) == 6 * 8 * 10240 * 4          # not served by the streaming kernel: split large-batch kernel
    dev = torch.device("cuda:0")
    P, h, h_kv, D, d_model, T = 8, 64, 8, 128, 8192, 20
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    x = torch.randn((T, d_model), device=dev, generator=g).to(torch.bfloat16)
    w = torch.randn(((h + 2 * h_kv) * D, d_model), device=dev, generator=g).to(torch.bfloat16)
    full = torch.empty(B.proj_workspace_bytes(T, w.shape[0], d_model), dtype=torch.uint8, device=dev)
    guard = torch.full((4096,), 0x77, dtype=torch.uint8, device=dev)
    short = guard[:1024]
    a = torch.empty((P, T, h // P + 2, D), dtype=torch.bfloat16, device=dev)
    b = torch.empty_like(a)
    c = torch.empty_like(a)
    B.qkv_proj_pack(x, w, a, P, h, h_kv, workspace=full)
    B.qkv_proj_pack(x, w, b, P, h, h_kv, workspace=short)
    B.qkv_proj_pack(x, w, c, P, h, h_kv)
    torch.cuda.synchronize()
    assert bool((guard == 0x77).all())
    assert torch.equal(b.view(torch.uint8), c.view(torch.uint8))
    assert torch.allclose(a.float(), c.float(), rtol=2.0 ** -7, atol=0.5)
