"""GPU parity of the FP8 E4M3 projections (Sec. 4.1 serves FP8 models; the scale rule is this library's reading) against
the CPU oracle, through the C ABI.

Quantisation: floating point decides integer codes, so both sides decide in float32 (maximum, amax / 448, x / scale) and
codes and scales are compared bit for bit.

Projection: the kernel and the oracle start from the same codes and scales.  The oracle sums the exact products in
float64.  The FP8 matrix-core instruction does not: it adds the 64 products of one instruction in small groups whose
members are aligned to the group's largest product with about 13 bits kept below it (probed on the chip: next to a
cancelling pair of products of 2^8, products of 2^-5 survive and products of 2^-6 vanish - six of them, the rest of an
8-product group).  A dropped or truncated product costs at most 2^-13 of its group's largest, so at most 8 * 2^-13 of the
sum of the group's magnitudes; the fp32 additions between instructions and the two scale multiplications are far below
that, and the final rounding to bf16 costs 2^-9 relative.  Bound used: |err| <= 2^-8 |ref| + 2^-9 * sum_k |term_k|
(twice the group bound)."""
import numpy as np
import pytest

from paper_2509_16495_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_backend
    return gpu_backend


def _bf16(rng, shape, scale=1.0):
    return W.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(scale))


def _dev_u8(G, a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(G.DEV)


def _dev_f32(G, a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(G.DEV)


def _check(got_bits, want, abs_terms):
    """abs_terms: sum over k of |term| for every output, in the output's units (bounds the error of the matrix core's sum)."""
    got = W.to_f64(got_bits, "bf16")
    assert got.shape == want.shape and np.all(np.isfinite(got))
    err = np.abs(got - want)
    bound = 2.0 ** -8 * np.abs(want) + 2.0 ** -9 * abs_terms + 1e-30
    assert np.all(err <= bound), float((err / bound).max())


@pytest.mark.parametrize("rows,cols", [(5, 64), (300, 512), (33, 8192), (2, 20480), (7, 8)])
def test_row_quantiser_bit_exact(oracle, G, rows, cols):
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(301))
    x = _bf16(rng, (rows, cols), 3.0)
    x[1] = 0                                             # a zero row
    x[0, ::3] = W.f32_to_bf16_bits(np.float32(1e-4) * np.ones(len(x[0, ::3]), dtype=np.float32))
    want_codes, want_scales = oracle.quantize_rows_e4m3(x, "bf16")
    codes = torch.full((rows, cols), 0x55, dtype=torch.uint8, device=G.DEV)
    scales = torch.zeros(rows, dtype=torch.float32, device=G.DEV)
    B.quantize_rows_fp8(G.t(x, "bf16"), codes, scales)
    torch.cuda.synchronize()
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), want_scales.view(np.uint32))
    assert np.array_equal(codes.cpu().numpy(), want_codes)


@pytest.mark.parametrize("P,hq_l,T,T_pad", [(8, 8, 37, 40), (4, 10, 5, 8), (1, 2, 3, 3)])
def test_recv_quantiser_bit_exact(oracle, G, P, hq_l, T, T_pad):
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(302))
    D = 128
    recv = _bf16(rng, (P, T_pad, hq_l, D), 0.7)
    rows = oracle.recv_rows(recv, T)
    want_codes, want_scales = oracle.quantize_rows_e4m3(rows, "bf16")
    codes = torch.full((P, T_pad, hq_l, D), 0x55, dtype=torch.uint8, device=G.DEV)
    scales = torch.zeros(T, dtype=torch.float32, device=G.DEV)
    B.quantize_recv_fp8(G.t(recv, "bf16"), codes, scales)
    torch.cuda.synchronize()
    got = codes.cpu().numpy()
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), want_scales.view(np.uint32))
    assert np.array_equal(oracle.recv_rows(got, T), want_codes)
    assert np.all(got[:, T:] == 0x55)                    # padding rows are left alone


QKV_CASES = [
    # P, h, h_kv, d_model, T, T_pad
    (8, 32, 8, 512, 300, 304),
    (8, 32, 4, 256, 70, 72),       # replication into several send buffers
    (4, 40, 8, 320, 257, 260),     # d_model no multiple of 128: five k tiles
    (1, 2, 1, 64, 5, 5),           # one k tile
    (2, 8, 4, 1024, 600, 600),
    (2, 8, 4, 192, 9, 10),         # three k tiles: fewer than the ring holds
    (8, 64, 8, 192, 0, 8),         # padding rows only
    (8, 8, 8, 5120, 20, 24),       # few output tiles, long k no multiple of 1024: with a workspace, k split over workgroups
    (8, 32, 8, 2048, 130, 136),
    (8, 8, 8, 8192, 8, 8),         # a decode step's few rows: the weight-streaming kernel (one pass over the codes)
    (8, 8, 8, 4096, 20, 24),       # two token blocks, one k group
    (8, 8, 8, 4096, 40, 40),       # four token blocks: two k groups with a workspace, the large-batch kernel without
    (4, 40, 8, 1024, 5, 8),        # 28 features per workgroup, one step per wavefront
    (8, 32, 4, 2048, 3, 4),        # replication into several send buffers
    (2, 4, 2, 2112, 100, 100),     # k split over two workgroups with a half-filled last stage in the second range
]


def _with_and_without_workspace(cases, k_of, rows_of):
    """Every case with a workspace; without one where that is another path (the oracle's part dominates the big ones)."""
    out = []
    for c in cases:
        out.append(c + (True,))
        if k_of(c) < 4096 or rows_of(c) > 32:
            out.append(c + (False,))
    return out


@pytest.mark.parametrize("P,h,h_kv,d_model,T,T_pad,give_workspace",
                         _with_and_without_workspace(QKV_CASES, lambda c: c[3], lambda c: c[5]))
def test_qkv_projection_fp8(oracle, G, P, h, h_kv, d_model, T, T_pad, give_workspace):
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(303))
    D = 128
    xc, xs = oracle.quantize_rows_e4m3(_bf16(rng, (max(T, 1), d_model)), "bf16")
    xc, xs = xc[:T], xs[:T]
    wc, ws = oracle.quantize_rows_e4m3(_bf16(rng, ((h + 2 * h_kv) * D, d_model), 0.05), "bf16")
    want = oracle.qkv_proj_pack_fp8(xc, xs, wc, ws, P, h, h_kv, D, T_pad)
    tab = np.abs(oracle.e4m3_table())
    tab[np.isnan(tab)] = 0.0
    terms = (tab[xc] @ tab[wc].T) * xs.astype(np.float64)[:, None] * ws.astype(np.float64)[None, :]
    terms = oracle.pack_heads_f64(terms.reshape(T, h + 2 * h_kv, D), P, h, h_kv, T_pad)
    send = torch.empty((P, T_pad, h // P + 2 * B.local_kv_heads(P, h_kv), D), dtype=torch.bfloat16, device=G.DEV)
    send.view(torch.uint8).fill_(0x55)
    ws_dev = None
    if give_workspace:
        ws_dev = torch.empty(max(B.proj_workspace_bytes(T_pad, (h + 2 * h_kv) * D, d_model, fp8=True), 16), dtype=torch.uint8, device=G.DEV)
    B.qkv_proj_pack_fp8(_dev_u8(G, xc).reshape(T, d_model), _dev_f32(G, xs), _dev_u8(G, wc), _dev_f32(G, ws), send, P, h, h_kv,
                        workspace=ws_dev)
    torch.cuda.synchronize()
    got = B.to_host(send)
    _check(got, want, terms)
    assert not np.any(got[:, T:])


O_CASES = [(8, 4, 512, 300, 304), (4, 10, 256, 257, 260), (1, 2, 256, 5, 5), (2, 4, 768, 600, 600), (8, 8, 256, 0, 4),
           (8, 4, 4096, 40, 40), (4, 8, 1024, 9, 12), (8, 4, 2048, 16, 16), (8, 8, 2048, 64, 64), (2, 4, 1024, 1, 1)]


@pytest.mark.parametrize("P,hq_l,d_model,T,T_pad,give_workspace",
                         _with_and_without_workspace(O_CASES, lambda c: c[0] * c[1] * 128, lambda c: c[3]))
def test_o_projection_fp8(oracle, G, P, hq_l, d_model, T, T_pad, give_workspace):
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(304))
    D = 128
    K = P * hq_l * D
    rc, rs = oracle.quantize_rows_e4m3(_bf16(rng, (max(T, 1), K)), "bf16")
    rc, rs = rc[:T], rs[:T]
    recv_codes = rng.integers(0, 0x7F, size=(P, T_pad, hq_l, D), dtype=np.uint8)     # padding rows hold arbitrary finite codes
    for p in range(P):
        recv_codes[p, :T] = rc[:, p * hq_l * D:(p + 1) * hq_l * D].reshape(T, hq_l, D)
    wc, ws = oracle.quantize_rows_e4m3(_bf16(rng, (d_model, K), 0.05), "bf16")
    want = oracle.unpack_o_proj_fp8(recv_codes, rs, wc, ws, T)
    tab = np.abs(oracle.e4m3_table())
    tab[np.isnan(tab)] = 0.0
    terms = (tab[rc] @ tab[wc].T) * rs.astype(np.float64)[:, None] * ws.astype(np.float64)[None, :]
    out = torch.empty((T, d_model), dtype=torch.bfloat16, device=G.DEV)
    out.view(torch.uint8).fill_(0x55)
    ws_dev = None
    if give_workspace:
        ws_dev = torch.empty(max(B.proj_workspace_bytes(T, d_model, K, fp8=True), 16), dtype=torch.uint8, device=G.DEV)
    B.unpack_o_proj_fp8(_dev_u8(G, recv_codes), _dev_f32(G, rs), _dev_u8(G, wc), _dev_f32(G, ws), out, workspace=ws_dev)
    torch.cuda.synchronize()
    _check(B.to_host(out), want, terms)


def test_quantise_then_project_stays_close_to_the_bf16_projection(oracle, G):
    """End to end on the GPU: quantiser + FP8 projection against the oracle's unquantised projection of the same bf16
    inputs; E4M3 keeps 4 significant bits per operand, so a sum of K products is off by about 2^-4.5 of its root-sum-square."""
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(305))
    P, h, h_kv, D, d_model, T = 8, 32, 8, 128, 1024, 200
    x, w = _bf16(rng, (T, d_model)), _bf16(rng, ((h + 2 * h_kv) * D, d_model), 0.03)
    xd, wd = G.t(x, "bf16"), G.t(w, "bf16")
    xq, xs = torch.empty((T, d_model), dtype=torch.uint8, device=G.DEV), torch.empty(T, dtype=torch.float32, device=G.DEV)
    wq, ws = torch.empty(w.shape, dtype=torch.uint8, device=G.DEV), torch.empty(w.shape[0], dtype=torch.float32, device=G.DEV)
    B.quantize_rows_fp8(xd, xq, xs)
    B.quantize_rows_fp8(wd, wq, ws)
    send = torch.empty((P, T, h // P + 2, D), dtype=torch.bfloat16, device=G.DEV)
    B.qkv_proj_pack_fp8(xq, xs, wq, ws, send, P, h, h_kv)
    torch.cuda.synchronize()
    got = W.to_f64(B.to_host(send), "bf16")
    want = oracle.qkv_proj_pack(x, w, P, h, h_kv, D, T, "bf16")
    rel = np.sqrt(np.mean((got - want) ** 2)) / np.sqrt(np.mean(want ** 2))
    assert rel < 0.06, rel


def test_full_size_70b_fp8_projections_on_sampled_rows(oracle, G):
    """The shapes the benchmark times (16384 tokens, d_model 8192, 64 + 2 x 8 heads, 8 buffers), quantised on the GPU:
    codes and scales of sampled token rows and weight rows bit-exact against the oracle's quantiser, and the outputs of
    those tokens for those features against the oracle's FP8 projection of its own codes."""
    import torch
    from paper_2509_16495_amd import binding as B
    rng = np.random.Generator(np.random.PCG64(306))
    P, h, h_kv, D, d_model, T = 8, 64, 8, 128, 8192, 16384
    hq_l, hkv_l = h // P, h_kv // P
    tokens = np.unique(np.concatenate([[0, 1, 127, 128, 255, 256, 257, 8191, 8192, 16127, 16128, 16383], rng.integers(0, T, 8)]))
    heads = [0, 1, 13, 63, h, h + 7, h + h_kv, h + 2 * h_kv - 1]       # q heads, first / last k head, first / last v head
    feats = np.concatenate([np.arange(j * D, (j + 1) * D) for j in heads])
    tok_d, feat_d = torch.from_numpy(tokens).to(G.DEV), torch.from_numpy(feats).to(G.DEV)
    tab = oracle.e4m3_table()
    atab = np.abs(tab)
    atab[np.isnan(atab)] = 0.0
    x, w = _bf16(rng, (T, d_model)), _bf16(rng, ((h + 2 * h_kv) * D, d_model), 0.02)
    xd, wd = G.t(x, "bf16"), G.t(w, "bf16")
    xq, xs = torch.empty(x.shape, dtype=torch.uint8, device=G.DEV), torch.empty(T, dtype=torch.float32, device=G.DEV)
    wq, ws = torch.empty(w.shape, dtype=torch.uint8, device=G.DEV), torch.empty(w.shape[0], dtype=torch.float32, device=G.DEV)
    B.quantize_rows_fp8(xd, xq, xs)
    B.quantize_rows_fp8(wd, wq, ws)
    send = torch.empty((P, T, hq_l + 2 * hkv_l, D), dtype=torch.bfloat16, device=G.DEV)
    send.view(torch.uint8).fill_(0x55)
    B.qkv_proj_pack_fp8(xq, xs, wq, ws, send, P, h, h_kv)
    torch.cuda.synchronize()
    xc_want, xs_want = oracle.quantize_rows_e4m3(x[tokens], "bf16")
    wc_want, ws_want = oracle.quantize_rows_e4m3(w[feats], "bf16")
    assert np.array_equal(xq[tok_d].cpu().numpy(), xc_want) and np.array_equal(xs[tok_d].cpu().numpy(), xs_want)
    assert np.array_equal(wq[feat_d].cpu().numpy(), wc_want) and np.array_equal(ws[feat_d].cpu().numpy(), ws_want)
    # the oracle on the sampled rows as a problem of its own (one buffer, the sampled heads as query heads): plain y[t][head][D]
    want = oracle.qkv_proj_pack_fp8(xc_want, xs_want, wc_want, ws_want, 1, len(heads), 0, D, len(tokens))[0]
    terms = ((atab[xc_want] @ atab[wc_want].T) * xs_want.astype(np.float64)[:, None] * ws_want.astype(np.float64)[None, :]).reshape(want.shape)
    got_all = B.to_host(send[:, tok_d].contiguous())                  # [P, tokens, hq_l + 2 hkv_l, D]
    got = np.empty((len(tokens), len(heads), D), dtype=got_all.dtype)
    for i, j in enumerate(heads):                                      # where the exchange layout puts head j (Sec. 3.2.1)
        if j < h:
            got[:, i] = got_all[j // hq_l, :, j % hq_l]
        elif j < h + h_kv:
            g = j - h
            got[:, i] = got_all[g // hkv_l, :, hq_l + g % hkv_l]
        else:
            g = j - h - h_kv
            got[:, i] = got_all[g // hkv_l, :, hq_l + hkv_l + g % hkv_l]
    _check(got, want, terms)
    del send, xd, wd, xq, wq, x, w
    # output projection: quantised out of the receive buffers; sampled output features
    recv, w_o = _bf16(rng, (P, T, hq_l, D)), _bf16(rng, (d_model, h * D), 0.02)
    cols = np.unique(np.concatenate([[0, 1, 127, 128, 255, 256, 4095, 4096, 8191], rng.integers(0, d_model, 200)]))
    col_d = torch.from_numpy(cols).to(G.DEV)
    rd, wod = G.t(recv, "bf16"), G.t(w_o, "bf16")
    rq, rs = torch.empty(recv.shape, dtype=torch.uint8, device=G.DEV), torch.empty(T, dtype=torch.float32, device=G.DEV)
    woq, wos = torch.empty(w_o.shape, dtype=torch.uint8, device=G.DEV), torch.empty(d_model, dtype=torch.float32, device=G.DEV)
    B.quantize_recv_fp8(rd, rq, rs)
    B.quantize_rows_fp8(wod, woq, wos)
    out = torch.empty((T, d_model), dtype=torch.bfloat16, device=G.DEV)
    out.view(torch.uint8).fill_(0x55)
    B.unpack_o_proj_fp8(rq, rs, woq, wos, out)
    torch.cuda.synchronize()
    rows = oracle.recv_rows(np.ascontiguousarray(recv[:, tokens]), len(tokens))
    rc_want, rs_want = oracle.quantize_rows_e4m3(rows, "bf16")
    woc_want, wos_want = oracle.quantize_rows_e4m3(w_o[cols], "bf16")
    assert np.array_equal(oracle.recv_rows(rq[:, tok_d].cpu().numpy(), len(tokens)), rc_want) and np.array_equal(rs[tok_d].cpu().numpy(), rs_want)
    assert np.array_equal(woq[col_d].cpu().numpy(), woc_want) and np.array_equal(wos[col_d].cpu().numpy(), wos_want)
    recv_codes = np.zeros((P, len(tokens), hq_l, D), dtype=np.uint8)
    for p in range(P):
        recv_codes[p] = rc_want[:, p * hq_l * D:(p + 1) * hq_l * D].reshape(len(tokens), hq_l, D)
    want_o = oracle.unpack_o_proj_fp8(recv_codes, rs_want, woc_want, wos_want, len(tokens))
    terms_o = (atab[rc_want] @ atab[woc_want].T) * rs_want.astype(np.float64)[:, None] * wos_want.astype(np.float64)[None, :]
    _check(B.to_host(out[tok_d][:, col_d].contiguous()), want_o, terms_o)
