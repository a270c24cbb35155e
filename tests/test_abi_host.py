"""Host-side checks of the C ABI (no GPU): the library loads, exports every function the header
declares, its index helpers reproduce the paper's worked examples, and every invalid-argument
path returns an error code before anything could be launched."""
import ast
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "shiftattn.h")


@pytest.fixture(scope="module")
def B():
    from paper_2509_16495_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2509_16495_amd import build
        build.build_library()
    binding.lib()
    return binding


def _declared_functions():
    """Every function declared in any header under include/."""
    import glob
    names = set()
    for header in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(shiftattn_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(B):
    names = _declared_functions()
    assert {"shiftattn_pack_seq2head", "shiftattn_prefill", "shiftattn_decode", "shiftattn_unpack_head2seq",
            "shiftattn_kv_write", "shiftattn_last_error"} <= set(names)
    for n in names:
        assert hasattr(B.lib(), n), n


def test_options_and_their_bounds(B):
    """The tuning switches: defaults are 0, values are range-checked, unknown options refused."""
    L = B.lib()
    for opt in (B.OPT_PREFILL_TILE, B.OPT_PREFILL_SPLITS, B.OPT_GENERIC_ONLY, B.OPT_PREFILL_PAIRING, B.OPT_PREFILL_SCALED_Q):
        assert B.get_option(opt) == 0
    assert L.shiftattn_set_option(B.OPT_PREFILL_SCALED_Q, 2) == B.EINVAL
    assert L.shiftattn_set_option(B.OPT_PREFILL_PAIRING, 3) == B.EINVAL and L.shiftattn_set_option(B.OPT_PREFILL_PAIRING, -1) == B.EINVAL
    assert L.shiftattn_set_option(B.OPT_PREFILL_TILE, 64) == B.EINVAL
    assert L.shiftattn_set_option(B.OPT_PREFILL_SPLITS, 65) == B.EINVAL and L.shiftattn_set_option(B.OPT_PREFILL_SPLITS, -1) == B.EINVAL
    assert L.shiftattn_set_option(B.OPT_GENERIC_ONLY, 2) == B.EINVAL
    assert L.shiftattn_set_option(17, 0) == B.EINVAL and B.get_option(17) == -1
    a = _attn(B, max_blocks_per_seq=8320)
    auto = B.prefill_workspace_bytes(1, 2048, 2048, 133120, a)
    try:
        B.set_option(B.OPT_PREFILL_SPLITS, 4)
        assert B.get_option(B.OPT_PREFILL_SPLITS) == 4
        assert B.prefill_workspace_bytes(1, 2048, 2048, 133120, a) == 4 * 2048 * 8 * (128 + 2) * 4   # sizes follow the switch
        B.set_option(B.OPT_GENERIC_ONLY, 1)
        assert B.prefill_workspace_bytes(1, 2048, 2048, 133120, a) == 0 and B.decode_workspace_bytes(4, 64, a) == 0
    finally:
        for opt in (B.OPT_PREFILL_TILE, B.OPT_PREFILL_SPLITS, B.OPT_GENERIC_ONLY, B.OPT_PREFILL_PAIRING, B.OPT_PREFILL_SCALED_Q):
            B.set_option(opt, 0)
    assert B.prefill_workspace_bytes(1, 2048, 2048, 133120, a) == auto


def test_launch_plans_follow_the_shape_of_the_batch(B):
    """Host logic behind the workspace queries (no GPU work): how many key ranges a prefill launch takes, seen through
    the size of its partial results, `ranges x rows x heads x (128 + 2) x 4` bytes; and the k ranges / k groups of the
    projections.  Shapes: the benchmark's batches (Table 4 head geometries on 8 ranks)."""
    def ranges(num_seqs, total_q, max_q, max_ctx, hq):
        a = _attn(B, num_q_heads=hq, max_blocks_per_seq=(max_ctx + 15) // 16)
        ws = B.prefill_workspace_bytes(num_seqs, total_q, max_q, max_ctx, a)
        assert ws % (total_q * hq * 130 * 4) == 0
        return ws // (total_q * hq * 130 * 4)

    assert ranges(4, 16384, 4096, 4096, 4) == 0         # 256 equal workgroups of 128-column tiles: one round, no split
    assert ranges(1, 16384, 16384, 16384, 8) == 0       # 256 pairs of 256-column tiles
    assert ranges(1, 2048, 2048, 133120, 8) == 4        # 64 tiles, one per workgroup (nothing to level by pairing): four ranges fill the chip
    assert ranges(1, 16384, 16384, 16384, 5) == 2       # 322 tiles, one per workgroup, heaviest first: two ranges bring the heaviest under a compute unit's share
    assert ranges(4, 16384, 4096, 4096, 5) == 0         # short contexts: the merge would cost more than the ragged round
    try:
        B.set_option(B.OPT_PREFILL_TILE, 128)
        assert ranges(1, 2048, 2048, 133120, 8) == 4    # 64 pairs of 128-column tiles
        B.set_option(B.OPT_PREFILL_TILE, 256)
        assert ranges(4, 16384, 4096, 4096, 4) == 2     # 128 pairs of 256-column tiles
        B.set_option(B.OPT_PREFILL_PAIRING, 1)
        assert ranges(1, 2048, 2048, 133120, 8) == 8    # in pairs the chunk is 32 workgroups: eight ranges fill the chip
        assert ranges(1, 16384, 16384, 16384, 5) == 3   # 161 pairs: three ranges make two full rounds
        B.set_option(B.OPT_PREFILL_PAIRING, 2)
        assert ranges(1, 16384, 16384, 16384, 8) == 0   # 512 tiles, heaviest first: the light ones level the chip out
    finally:
        B.set_option(B.OPT_PREFILL_TILE, 0)
        B.set_option(B.OPT_PREFILL_PAIRING, 0)
    # projections: k groups of the streaming kernel (token slice of a wavefront <= 128 registers), k ranges of the
    # large-batch kernel while its tiles are few, nothing once they fill the chip
    n, k = 10240, 8192
    assert [B.proj_workspace_bytes(t, n, k) // (n * 4) for t in (1, 16, 17, 32, 33, 64)] == [0, 0, 2 * 32, 2 * 32, 4 * 64, 4 * 64]
    assert B.proj_workspace_bytes(65, n, k) == 6 * 65 * n * 4 and B.proj_workspace_bytes(512, n, k) == 3 * 512 * n * 4
    assert B.proj_workspace_bytes(1024, n, k) == 0 and B.proj_workspace_bytes(16384, n, k) == 0
    # 2048 rows are 320 tiles: six token tiles whole (240 tiles), the last 512 rows in three k ranges (240 work items)
    assert B.proj_workspace_bytes(2048, n, k) == 3 * 512 * n * 4
    assert B.proj_workspace_bytes(8, 6144, 4096) == 0 and B.proj_workspace_bytes(0, n, k) == 0
    # whatever the plan, the workspace is whole fp32 rows of the result: at most 16 ranges of at most all rows, rows of
    # whole leading tiles excluded in steps of 256, and nothing when the tiles are a whole number of rounds of the chip
    for feats, kk in ((10240, 8192), (8192, 8192), (6144, 4096), (2560, 5120), (256, 64)):
        for rows in (65, 100, 255, 256, 257, 511, 777, 1024, 1500, 2048, 2300, 4096, 5000, 8192, 16384, 20000):
            for fp8 in (False, True):
                need = B.proj_workspace_bytes(rows, feats, kk, fp8=fp8)
                assert need % (feats * 4) == 0
                q = need // (feats * 4)   # ranges x rows they cover
                assert q <= 16 * rows
                if q:
                    covered = [r for r in range(rows, 0, -256) if q % r == 0 and 2 <= q // r <= 16]
                    assert covered, (rows, feats, kk, q)
                if (feats // 256) * (-(-rows // 256)) % 256 == 0:
                    assert need == 0, (rows, feats, kk)


def test_struct_layouts_match_header(B):
    assert ctypes.sizeof(B.Xchg) == 20
    assert ctypes.sizeof(B.Attn) == 72 and B.Attn.q_stride.offset == 32 and B.Attn.kv_format.offset == 56


def test_head_block_matches_paper_example(B):
    gold = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "process_groups_sp3_tp2.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split("=", 1)
            gold[k.strip()] = ast.literal_eval(v.strip())
    sp, tp = gold["SP"], gold["TP"]
    blocks = [B.head_block(sp, tp, r) for r in range(sp * tp)]
    for rank, head in gold["HEAD_OF_RANK"].items():
        assert blocks[rank] == head
    assert [blocks.index(b) for b in range(sp * tp)] == gold["SP_TP_GROUP"][0]
    assert B.head_block(3, 2, 6) == -1 and B.head_block(0, 2, 0) == -1 and B.head_block(3, 2, -1) == -1


def test_shift_dispatcher_threshold(B):
    """Algorithm 2: batches larger than the threshold run in the base configuration, the rest in the
    shift configuration."""
    assert B.use_base_config(4097, 4096) == 1 and B.use_base_config(4096, 4096) == 0 and B.use_base_config(0, 0) == 0
    assert B.use_base_config(1, 0) == 1 and B.use_base_config(-1, 5) == -1 and B.use_base_config(5, -1) == -1


def test_replication_and_padding_helpers(B):
    assert [B.kv_head_of_block(p, 8, 4) for p in range(8)] == [0, 0, 1, 1, 2, 2, 3, 3]
    assert [B.kv_head_of_block(p, 4, 8) for p in range(4)] == [0, 2, 4, 6]
    assert B.kv_head_of_block(8, 8, 4) == -1
    assert B.padded_tokens(9, 8) == 16 and B.padded_tokens(16, 8) == 16 and B.padded_tokens(0, 8) == 0
    assert B.padded_tokens(-1, 8) == -1 and B.padded_tokens(5, 0) == -1


def _xchg(B, **kw):
    d = dict(P=2, num_q_heads=8, num_kv_heads=0, head_dim=64, dtype=B.F32)
    d.update(kw)
    return B.Xchg(d["P"], d["num_q_heads"], d["num_kv_heads"], d["head_dim"], d["dtype"])


def _attn(B, **kw):
    d = dict(num_q_heads=8, num_kv_heads=1, head_dim=128, dtype=B.BF16, block_size=16, num_blocks=64,
             max_blocks_per_seq=8, softmax_scale=0.1, q_stride=0, kv_stride=0, out_stride=0, kv_format=0, k_scale=0.0,
             v_scale=0.0, reserved=0)
    d.update(kw)
    return B.Attn(*[d[f[0]] for f in B.Attn._fields_])


FAKE = ctypes.c_void_p(0x1000)  # aligned, never dereferenced: every case below fails validation first


def test_pack_unpack_reject_bad_arguments(B):
    L = B.lib()
    cases = [
        (dict(P=0), 4, 4, B.EINVAL), (dict(P=3), 4, 4, B.EINVAL), (dict(num_kv_heads=3, P=2), 4, 4, B.EINVAL),
        (dict(dtype=7), 4, 4, B.EINVAL), (dict(), 5, 4, B.EINVAL), (dict(), -1, 4, B.EINVAL),
        (dict(head_dim=6), 4, 4, B.EUNSUPPORTED), (dict(head_dim=0), 4, 4, B.EINVAL),
        (dict(num_q_heads=12, num_kv_heads=6, P=4), 4, 4, B.EINVAL),
    ]
    for kw, T, T_pad, code in cases:
        x = _xchg(B, **kw)
        assert L.shiftattn_pack_seq2head(FAKE, FAKE, T, T_pad, ctypes.byref(x), None) == code, kw
        assert B.last_error()
    x = _xchg(B)
    assert L.shiftattn_pack_seq2head(None, FAKE, 4, 4, ctypes.byref(x), None) == B.EINVAL
    assert L.shiftattn_pack_seq2head(FAKE, None, 4, 4, ctypes.byref(x), None) == B.EINVAL
    assert L.shiftattn_pack_seq2head(ctypes.c_void_p(0x1008), FAKE, 4, 4, ctypes.byref(x), None) == B.EINVAL
    assert L.shiftattn_pack_seq2head(FAKE, FAKE, 4, 4, None, None) == B.EINVAL
    assert L.shiftattn_unpack_head2seq(None, FAKE, 4, 4, ctypes.byref(x), None) == B.EINVAL
    assert L.shiftattn_unpack_head2seq(FAKE, FAKE, 4, 3, ctypes.byref(x), None) == B.EINVAL
    # empty problems are valid no-ops and touch nothing
    assert L.shiftattn_pack_seq2head(None, None, 0, 0, ctypes.byref(x), None) == B.OK
    assert L.shiftattn_unpack_head2seq(None, None, 0, 4, ctypes.byref(x), None) == B.OK
    big = _xchg(B, num_q_heads=1 << 20, P=1, head_dim=256)
    assert L.shiftattn_pack_seq2head(FAKE, FAKE, 1 << 20, 1 << 20, ctypes.byref(big), None) == B.EUNSUPPORTED


def test_attention_entry_points_reject_bad_arguments(B):
    L = B.lib()

    def prefill(a, q=FAKE, k=None, v=None, slots=None, cache=FAKE, table=FAKE, cu=FAKE, sl=FAKE, S=1, tq=32, mq=32,
                ms=64, out=FAKE, ws=None, wsb=0):
        return L.shiftattn_prefill(q, k, v, slots, cache, table, cu, sl, S, tq, mq, ms, out, ws, wsb,
                                   None if a is None else ctypes.byref(a), None)

    def decode(a, q=FAKE, k=None, v=None, slots=None, cache=FAKE, table=FAKE, sl=FAKE, S=4, ms=64, out=FAKE, ws=None,
               wsb=0):
        return L.shiftattn_decode(q, k, v, slots, cache, table, sl, S, ms, out, ws, wsb,
                                  None if a is None else ctypes.byref(a), None)

    ok = _attn(B)
    assert prefill(None) == B.EINVAL and decode(None) == B.EINVAL
    for kw, code in [(dict(num_kv_heads=3), B.EINVAL), (dict(num_kv_heads=0), B.EINVAL), (dict(dtype=5), B.EINVAL),
                     (dict(head_dim=100), B.EUNSUPPORTED), (dict(head_dim=512), B.EUNSUPPORTED),
                     (dict(block_size=32), B.EUNSUPPORTED), (dict(softmax_scale=0.0), B.EINVAL),
                     (dict(softmax_scale=-1.0), B.EINVAL), (dict(softmax_scale=float("nan")), B.EINVAL),
                     (dict(q_stride=100), B.EINVAL), (dict(kv_stride=8), B.EINVAL), (dict(out_stride=1028), B.EINVAL),
                     (dict(max_blocks_per_seq=2), B.EINVAL), (dict(kv_format=7), B.EINVAL), (dict(reserved=1), B.EINVAL),
                     (dict(kv_format=B.KV_FP8_E4M3), B.EINVAL),  # scales missing
                     (dict(kv_format=B.KV_FP8_E4M3, k_scale=1.0, v_scale=-1.0), B.EINVAL),
                     (dict(kv_format=B.KV_FP8_E4M3, k_scale=float("inf"), v_scale=1.0), B.EINVAL),
                     (dict(kv_format=B.KV_FP8_E4M3, k_scale=1.0, v_scale=1.0, head_dim=72), B.EUNSUPPORTED)]:
        assert prefill(_attn(B, **kw)) == code, kw
        assert decode(_attn(B, **kw)) == code, kw
    for kw in (dict(q=None), dict(cache=None), dict(table=None), dict(sl=None), dict(out=None)):
        assert prefill(ok, **kw) == B.EINVAL and decode(ok, **kw) == B.EINVAL
    assert prefill(ok, cu=None) == B.EINVAL
    assert prefill(ok, k=FAKE) == B.EINVAL and decode(ok, v=FAKE, slots=FAKE) == B.EINVAL
    assert prefill(ok, q=ctypes.c_void_p(0x1002)) == B.EINVAL
    assert prefill(ok, S=-1) == B.EINVAL and prefill(ok, mq=64, tq=32) == B.EINVAL and prefill(ok, mq=128, tq=128, ms=64) == B.EINVAL
    assert decode(ok, S=-1) == B.EINVAL
    # decode always needs a workspace on the tuned path; a missing or short one is reported, not used
    need = B.decode_workspace_bytes(4, 64, ok)
    assert need > 0
    assert decode(ok) == B.EWORKSPACE and decode(ok, ws=FAKE, wsb=need - 1) == B.EWORKSPACE
    # the variant without a workspace argument: same argument checks; a batch beyond the library's own array is refused
    def decode_static(a, q=FAKE, cache=FAKE, table=FAKE, sl=FAKE, S=4, ms=64, out=FAKE):
        return L.shiftattn_decode_static(q, None, None, None, cache, table, sl, S, ms, out, None if a is None else ctypes.byref(a), None)

    assert decode_static(None) == B.EINVAL and decode_static(_attn(B, head_dim=100)) == B.EUNSUPPORTED
    assert decode_static(ok, S=-1) == B.EINVAL
    assert decode_static(ok, q=None, cache=None, table=None, sl=None, out=None, S=0, ms=0) == B.OK
    wide = _attn(B, num_q_heads=16)
    assert B.decode_workspace_bytes(2048, 64, wide) > B.STATIC_SCRATCH_BYTES
    assert decode_static(wide, S=2048) == B.EWORKSPACE and "scratch" in B.last_error()
    # split prefill (short chunk on a long context) needs one too
    long_ctx = _attn(B, max_blocks_per_seq=8320)
    need = B.prefill_workspace_bytes(1, 2048, 2048, 133120, long_ctx)
    assert need > 0
    assert prefill(long_ctx, tq=2048, mq=2048, ms=133120) == B.EWORKSPACE
    assert B.prefill_workspace_bytes(4, 16384, 4096, 4096, _attn(B, num_q_heads=4, max_blocks_per_seq=256)) == 0
    # empty batches are valid no-ops
    assert prefill(ok, q=None, cache=None, table=None, cu=None, sl=None, out=None, S=0, tq=0, mq=0, ms=0) == B.OK
    assert decode(ok, q=None, cache=None, table=None, sl=None, out=None, S=0, ms=0) == B.OK
    # unified batch: same checks, plus its own
    def mixed(a, q=FAKE, k=None, v=None, slots=None, cache=FAKE, table=FAKE, cu=FAKE, sl=FAKE, Sp=1, tq=32, mq=32, msp=64,
              Sd=4, msd=64, out=FAKE, ws=None, wsb=0):
        return L.shiftattn_mixed(q, k, v, slots, cache, table, cu, sl, Sp, tq, mq, msp, Sd, msd, out, ws, wsb,
                                 None if a is None else ctypes.byref(a), None)

    assert mixed(None) == B.EINVAL and mixed(ok, Sd=-1) == B.EINVAL and mixed(ok, Sp=0, tq=32) == B.EINVAL
    assert mixed(ok, q=None) == B.EINVAL and mixed(ok, cu=None) == B.EINVAL and mixed(ok, k=FAKE) == B.EINVAL
    assert mixed(ok) == B.EWORKSPACE  # the decode part needs one
    assert B.mixed_workspace_bytes(1, 32, 32, 64, 4, 64, ok) == B.decode_workspace_bytes(4, 64, ok)
    assert B.mixed_workspace_bytes(1, 2048, 2048, 133120, 4, 64, long_ctx) == \
        max(B.prefill_workspace_bytes(1, 2048, 2048, 133120, long_ctx), B.decode_workspace_bytes(4, 64, long_ctx))
    assert mixed(ok, q=None, cache=None, table=None, cu=None, sl=None, out=None, Sp=0, tq=0, mq=0, msp=0, Sd=0, msd=0) == B.OK
    # a call that brings new K/V is refused as a whole, before its write is launched, when a part is bad
    need = B.mixed_workspace_bytes(1, 32, 32, 64, 4, 64, ok)
    small = _attn(B, max_blocks_per_seq=2)  # 32 tokens per sequence at most
    for bad in (dict(a=small, msp=32, msd=64), dict(a=small, msp=64, msd=32), dict(a=ok, mq=64), dict(a=ok, out=ctypes.c_void_p(0x1002))):
        a = bad.pop("a")
        assert mixed(a, k=FAKE, v=FAKE, slots=FAKE, ws=FAKE, wsb=need, **bad) == B.EINVAL, bad
    kvw = L.shiftattn_kv_write
    assert kvw(None, FAKE, FAKE, 4, FAKE, ctypes.byref(ok), None) == B.EINVAL
    assert kvw(FAKE, FAKE, FAKE, -1, FAKE, ctypes.byref(ok), None) == B.EINVAL
    assert kvw(None, None, None, 0, None, ctypes.byref(ok), None) == B.OK
    assert B.lib().shiftattn_decode_workspace_bytes(-1, 64, ctypes.byref(ok)) == ctypes.c_size_t(-1).value


def test_projection_entry_points_reject_bad_arguments(B):
    """The fused projections (Algorithm 1, the products next to the two all-to-alls): bf16, head_dim 128 only."""
    L = B.lib()
    ok = dict(P=8, num_q_heads=64, num_kv_heads=8, head_dim=128, dtype=B.BF16)
    x = _xchg(B, **ok)
    q, o = L.shiftattn_qkv_proj_pack, L.shiftattn_unpack_o_proj
    # shapes the GEMM is not built for
    for kw, d_model in [(dict(dtype=B.F32), 8192), (dict(head_dim=64), 8192), (dict(), 8200), (dict(num_q_heads=9, num_kv_heads=1, P=1), 8192)]:
        bad = _xchg(B, **{**ok, **kw})
        assert q(FAKE, FAKE, FAKE, 8, 8, d_model, ctypes.byref(bad), None) == B.EUNSUPPORTED, (kw, d_model)
        assert "projection" in B.last_error()
    for kw, d_model in [(dict(dtype=B.F32), 8192), (dict(head_dim=64), 8192), (dict(), 8192 + 64)]:
        bad = _xchg(B, **{**ok, **kw, "num_kv_heads": 0})
        assert o(FAKE, FAKE, FAKE, 8, 8, d_model, ctypes.byref(bad), None) == B.EUNSUPPORTED, (kw, d_model)
    xo = _xchg(B, **{**ok, "num_kv_heads": 0})
    # invalid arguments: sizes, descriptor, pointers, alignment
    for fn, desc in ((q, x), (o, xo)):
        assert fn(FAKE, FAKE, FAKE, 9, 8, 8192, ctypes.byref(desc), None) == B.EINVAL      # T > T_pad
        assert fn(FAKE, FAKE, FAKE, 8, 8, 0, ctypes.byref(desc), None) == B.EINVAL
        assert fn(FAKE, FAKE, FAKE, 8, 8, -64, ctypes.byref(desc), None) == B.EINVAL
        assert fn(FAKE, FAKE, FAKE, 8, 8, 8192, None, None) == B.EINVAL
        assert fn(None, FAKE, FAKE, 8, 8, 8192, ctypes.byref(desc), None) == B.EINVAL
        assert fn(FAKE, None, FAKE, 8, 8, 8192, ctypes.byref(desc), None) == B.EINVAL
        assert fn(FAKE, FAKE, None, 8, 8, 8192, ctypes.byref(desc), None) == B.EINVAL
        assert fn(FAKE, ctypes.c_void_p(0x1004), FAKE, 8, 8, 8192, ctypes.byref(desc), None) == B.EINVAL
        assert B.last_error()
    bad_p = _xchg(B, **{**ok, "P": 3})
    assert q(FAKE, FAKE, FAKE, 6, 6, 8192, ctypes.byref(bad_p), None) == B.EINVAL          # heads not divisible by P
    # the forms with a workspace: the same checks, and a workspace must exist and be aligned if a size is given
    qw, ow = L.shiftattn_qkv_proj_pack_ws, L.shiftattn_unpack_o_proj_ws
    for fn, desc in ((qw, x), (ow, xo)):
        assert fn(FAKE, FAKE, FAKE, 9, 8, 8192, ctypes.byref(desc), None, 0, None) == B.EINVAL
        assert fn(None, FAKE, FAKE, 8, 8, 8192, ctypes.byref(desc), None, 0, None) == B.EINVAL
        assert fn(FAKE, FAKE, FAKE, 32, 32, 8192, ctypes.byref(desc), None, 4096, None) == B.EINVAL and "workspace" in B.last_error()
        assert fn(FAKE, FAKE, FAKE, 32, 32, 8192, ctypes.byref(desc), ctypes.c_void_p(0x1004), 4096, None) == B.EINVAL
        assert fn(None, None, None, 0, 0, 8192, ctypes.byref(desc), None, 0, None) == B.OK
    assert L.shiftattn_proj_workspace_bytes(-1, 10240, 8192) == 0 and L.shiftattn_proj_workspace_bytes(8, 0, 8192) == 0
    # empty problems are valid no-ops and touch nothing
    assert q(None, None, None, 0, 0, 8192, ctypes.byref(x), None) == B.OK
    assert o(None, None, None, 0, 8, 8192, ctypes.byref(xo), None) == B.OK


def test_fp8_projection_entry_points_reject_bad_arguments(B):
    """Row quantiser and the projections over FP8 E4M3 codes: every case fails validation before anything is launched."""
    L = B.lib()
    ok = dict(P=8, num_q_heads=64, num_kv_heads=8, head_dim=128, dtype=B.BF16)
    x, xo = _xchg(B, **ok), _xchg(B, **{**ok, "num_kv_heads": 0})
    qr, qv, q8, o8 = L.shiftattn_quantize_rows_fp8, L.shiftattn_quantize_recv_fp8, L.shiftattn_qkv_proj_pack_fp8, L.shiftattn_unpack_o_proj_fp8
    assert qr(FAKE, FAKE, FAKE, -1, 64, None) == B.EINVAL and qr(FAKE, FAKE, FAKE, 4, 0, None) == B.EINVAL
    assert qr(FAKE, FAKE, FAKE, 4, 12, None) == B.EUNSUPPORTED                 # cols no multiple of 8
    assert qr(None, FAKE, FAKE, 4, 64, None) == B.EINVAL and qr(FAKE, None, FAKE, 4, 64, None) == B.EINVAL
    assert qr(FAKE, FAKE, None, 4, 64, None) == B.EINVAL
    assert qr(ctypes.c_void_p(0x1008), FAKE, FAKE, 4, 64, None) == B.EINVAL    # x not 16-byte aligned
    assert qr(FAKE, FAKE, ctypes.c_void_p(0x1002), 4, 64, None) == B.EINVAL    # scales not 4-byte aligned
    assert qr(None, None, None, 0, 64, None) == B.OK
    assert qv(FAKE, FAKE, FAKE, 9, 8, ctypes.byref(xo), None) == B.EINVAL      # T > T_pad
    assert qv(FAKE, FAKE, FAKE, 8, 8, ctypes.byref(_xchg(B, **{**ok, "dtype": B.F32, "num_kv_heads": 0})), None) == B.EUNSUPPORTED
    assert qv(FAKE, FAKE, FAKE, 8, 8, None, None) == B.EINVAL and qv(None, FAKE, FAKE, 8, 8, ctypes.byref(xo), None) == B.EINVAL
    assert qv(None, None, None, 0, 8, ctypes.byref(xo), None) == B.OK
    for kw, d_model in [(dict(dtype=B.F32), 8192), (dict(head_dim=64), 8192), (dict(), 8200), (dict(num_q_heads=9, num_kv_heads=1, P=1), 8192)]:
        bad = _xchg(B, **{**ok, **kw})
        assert q8(FAKE, FAKE, FAKE, FAKE, FAKE, 8, 8, d_model, ctypes.byref(bad), None) == B.EUNSUPPORTED, (kw, d_model)
    assert o8(FAKE, FAKE, FAKE, FAKE, FAKE, 8, 8, 8192 + 64, ctypes.byref(xo), None) == B.EUNSUPPORTED
    for fn, desc in ((q8, x), (o8, xo)):
        assert fn(FAKE, FAKE, FAKE, FAKE, FAKE, 9, 8, 8192, ctypes.byref(desc), None) == B.EINVAL
        assert fn(FAKE, FAKE, FAKE, FAKE, FAKE, 8, 8, 0, ctypes.byref(desc), None) == B.EINVAL
        assert fn(FAKE, FAKE, FAKE, FAKE, FAKE, 8, 8, 8192, None, None) == B.EINVAL
        for hole in range(5):
            args = [FAKE] * 5
            args[hole] = None
            assert fn(*args, 8, 8, 8192, ctypes.byref(desc), None) == B.EINVAL, hole
        assert fn(FAKE, ctypes.c_void_p(0x1002), FAKE, FAKE, FAKE, 8, 8, 8192, ctypes.byref(desc), None) == B.EINVAL
        assert fn(ctypes.c_void_p(0x1008), FAKE, FAKE, FAKE, FAKE, 8, 8, 8192, ctypes.byref(desc), None) == B.EINVAL
        assert B.last_error()
    assert q8(None, None, None, None, None, 0, 0, 8192, ctypes.byref(x), None) == B.OK
    assert o8(None, None, None, None, None, 0, 8, 8192, ctypes.byref(xo), None) == B.OK
