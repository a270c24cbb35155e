"""A whole step captured into a HIP graph and replayed (Sec. 3.4: the engine replays captured graphs for
both configurations, so every call of the path has to be capturable: no allocation, no synchronisation, no
host read of device memory).  Each replay is compared bit for bit with the eager result on the same inputs;
between replays the inputs' contents change (same buffers), and the program does eager work and
synchronises.
"""
import numpy as np
import pytest
import torch

from paper_2509_16495_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("fp8", [False, True])
def test_step_replays_match_eager(fp8):
    from paper_2509_16495_amd import binding as B
    import gpu_backend as G
    dev = G.DEV
    P, H, H_kv, D = 4, 16, 4, 128
    hq_l, hkv_l = H // P, 1
    seqs = [(200, 200), (64, 900), (1, 1), (33, 33)] + [(1, int(c)) for c in (5, 64, 777, 2000, 31)]
    n_pre = 4
    case = W.make_attn_case("graph", 90, "bf16", seqs, hq_l, hkv_l, D, pool_factor=1.5)
    n = case.total_q
    T = (n + P - 1) // P
    rng = np.random.Generator(np.random.PCG64(91))
    scales = (0.04, 0.03) if fp8 else (1.0, 1.0)

    def fused_rows(seed):
        r = np.random.Generator(np.random.PCG64(seed))
        return B.to_device(W.f32_to_bf16_bits(r.standard_normal((n, hq_l + 2 * hkv_l, D), dtype=np.float32)), "bf16", dev)

    qkv_local = B.to_device(W.f32_to_bf16_bits(rng.standard_normal((T, H + 2 * H_kv, D), dtype=np.float32)), "bf16", dev)
    send = torch.empty((P, T, hq_l + 2 * hkv_l, D), dtype=torch.bfloat16, device=dev)
    recv = fused_rows(1)                      # stands for the buffer the first exchange delivers
    attn_o = torch.zeros((n, hq_l, D), dtype=torch.bfloat16, device=dev)
    recv2 = torch.empty((P, T, hq_l, D), dtype=torch.bfloat16, device=dev)
    out_seq = torch.empty((T, H, D), dtype=torch.bfloat16, device=dev)
    cache0 = G.cache_for_case(case, only_cached=True, fp8_scales=scales if fp8 else None)
    cache = cache0.clone()
    table, cu, sl = G.ti(case.block_table, np.int32), G.ti(case.cu_seqlens_q[:n_pre + 1], np.int32), G.ti(case.ctx_lens, np.int32)
    slots = G.ti(case.slots[case.new_token_index], np.int64)
    q_v, k_v, v_v = recv[:, :hq_l], recv[:, hq_l:hq_l + hkv_l], recv[:, hq_l + hkv_l:]
    mq, msp, msd = int(case.q_lens[:n_pre].max()), int(case.ctx_lens[:n_pre].max()), int(case.ctx_lens[n_pre:].max())
    a = B.attn_desc(q_v, cache, table, case.softmax_scale, k_v, attn_o, *scales)
    ws = torch.empty(max(B.mixed_workspace_bytes(n_pre, int(case.q_lens[:n_pre].sum()), mq, msp, case.num_seqs - n_pre, msd, a), 16),
                     dtype=torch.uint8, device=dev)

    def step():
        B.pack_seq2head(qkv_local, send, P, H, H_kv)
        B.mixed(q_v, cache, table, cu, sl, n_pre, mq, msp, msd, attn_o, case.softmax_scale, k_new=k_v, v_new=v_v,
                slot_mapping=slots, workspace=ws, k_scale=scales[0], v_scale=scales[1])
        recv2.view(-1)[:n * hq_l * D].copy_(attn_o.view(-1))     # stands for the second exchange
        B.unpack_head2seq(recv2, out_seq)

    def snapshot():
        torch.cuda.synchronize()
        return [x.clone() for x in (send, attn_o, out_seq, cache)]

    step()                                    # warm-up outside the capture (one-time function attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        recv.copy_(fused_rows(100 + rep))     # new contents, same buffers
        qkv_local.copy_(torch.roll(qkv_local, 1, 0))
        cache.copy_(cache0)
        recv2.zero_()
        step()
        want = snapshot()
        cache.copy_(cache0)
        for x in (send, attn_o, out_seq):
            x.zero_()
        recv2.zero_()
        _ = (qkv_local.float() * 2).sum().item()   # eager work and a synchronisation between replays
        graph.replay()
        got = snapshot()
        for g_, w_ in zip(got, want):
            assert torch.equal(g_.view(torch.uint8), w_.view(torch.uint8)), rep
