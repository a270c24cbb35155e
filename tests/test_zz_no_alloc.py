"""shiftattn_decode_static (the entry point for callers that cannot allocate) against shiftattn_decode.

Both run the same kernels; the static variant keeps the split partials in the library's own device array.
Two calls in a row, the second on a smaller batch, each compared bit for bit with the ordinary entry point
on the same inputs (results are bitwise reproducible: the merge order is fixed), and the first also with
the fp64 oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2509_16495_amd import binding as B          # noqa: E402
from paper_2509_16495_amd import workloads as W        # noqa: E402
import gpu_backend as G                                # noqa: E402


def _run(case, static: bool):
    dt = case.dtype
    cache = G.cache_for_case(case, only_cached=True)
    fused = np.concatenate([case.q, case.k_ctx[case.new_token_index], case.v_ctx[case.new_token_index]], axis=1)
    ft = G.t(fused, dt)
    q = ft[:, :case.hq_l]
    kw = dict(k_new=ft[:, case.hq_l:case.hq_l + case.hkv_l], v_new=ft[:, case.hq_l + case.hkv_l:],
              slot_mapping=G.ti(case.slots[case.new_token_index], np.int64))
    out = torch.empty((case.num_seqs, case.hq_l, case.D), dtype=G.torch_dtype(dt), device=G.DEV)
    out.view(torch.uint8).fill_(0x5A)
    fn = B.decode_static if static else B.decode
    fn(q, cache, G.ti(case.block_table, np.int32), G.ti(case.ctx_lens, np.int32), int(case.ctx_lens.max()), out,
       case.softmax_scale, **kw)
    torch.cuda.synchronize()
    return B.to_host(out), B.to_host(cache)


def test_decode_static_matches_decode_twice_in_a_row(oracle):
    rng = np.random.Generator(np.random.PCG64(77))
    big = W.make_attn_case("static_big", 71, "bf16", [(1, int(c)) for c in rng.integers(40, 3000, size=48)], 8, 1, 128)
    small = W.make_attn_case("static_small", 72, "bf16", [(1, int(c)) for c in rng.integers(1, 700, size=5)], 8, 1, 128)
    for case in (big, small):       # second call: smaller batch, the array still holds the first call's partials
        got_s, cache_s = _run(case, static=True)
        got_d, cache_d = _run(case, static=False)
        assert got_s.tobytes() == got_d.tobytes(), case.name
        assert cache_s.tobytes() == cache_d.tobytes(), case.name
        want = oracle.attention_case(case, oracle.cache_for_case(case))
        err = np.abs(W.to_f64(got_s, "bf16") - want)
        assert err.max() <= 2e-2 and err.mean() <= 1e-3, (case.name, err.max(), err.mean())


def test_decode_static_refuses_batches_beyond_its_array():
    n = 2048
    q = torch.zeros((n, 16, 128), dtype=torch.bfloat16, device=G.DEV)
    cache = torch.zeros((4, 1, 2, 16 * 128), dtype=torch.bfloat16, device=G.DEV)
    table = torch.zeros((n, 1), dtype=torch.int32, device=G.DEV)
    sl = torch.ones(n, dtype=torch.int32, device=G.DEV)
    a = B.attn_desc(q, cache, table, 0.1, None, q)
    assert B.decode_workspace_bytes(n, 16, a) > B.STATIC_SCRATCH_BYTES
    with pytest.raises(B.ShiftAttnError) as ei:
        B.decode_static(q, cache, table, sl, 16, torch.empty_like(q), 0.1)
    assert ei.value.code == B.EWORKSPACE
