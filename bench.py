#!/usr/bin/env python3
"""Benchmark of one GPU's share of a Shift-Parallelism attention layer on MI355X.

A "step" is one pass of the whole hot path over one synthetic batch, with every input already in
HBM: send-side pack of this rank's fused QKV rows, causal prefill with fused KV-cache append,
receive-side unpack, and one decode step (with its KV append) for the same sequences.  The batch is
the Llama-3.1-8B-shaped shard at P=8 (4 query heads / 1 KV head, head_dim 128, 4 sequences of 4096
tokens, 16-token cache blocks in a random block-table permutation).  The wire exchange between the
ranks is not part of the path: the buffers it would deliver are staged in HBM beforehand.

One JSON line goes to stdout.  `value` is attention TFLOP/s of the whole step (4*D flops per
(query, visible key) pair per query head, masked pairs and softmax not counted, divided by the
wall time of the step).  `roofline` prices the dominant kernel (the MFMA prefill kernel) against
the chip's dense bf16 MFMA peak using HIP-event timing of that kernel alone.  `cpu_baseline` is the
fp64 CPU oracle timed on a stated sample of the same batch.  Further objects report the
HBM-bound kernels on the configurations that are large enough to measure bandwidth (batch decode of
256 sequences, exchange of a [16384, 64, 128] hidden state) and the 70B-shaped prefill.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def load_traffic():
    """HBM bytes per launch measured with rocprofv3 counters, from the committed summary table.

    Rows look like `| key | kernel | fetch bytes | write bytes | ...`; returns {key: fetch + write}."""
    out = {}
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) >= 4 and cells[0] and cells[0][0].isalpha():
                    try:
                        out[cells[0]] = int(float(cells[2])) + int(float(cells[3]))
                    except ValueError:
                        pass
    except OSError:
        pass
    return out
METRIC = "prefill attn TFLOP/s + decode KV-read GB/s per MI355X (head shard, % roofline)"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the decode / exchange / 70B-prefill configurations")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="also run a plain 1-GiB elementwise copy a few times (reference for scaling FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's share of the layer and runs on exactly one GPU; "
              f"--gpus {args.gpus} is not supported (no collectives are part of the path).", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2509_16495_amd import binding as B
    from paper_2509_16495_amd import workloads as W

    B.lib()  # fail loudly if the HIP library was not built
    traffic = load_traffic()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    bf = torch.bfloat16

    def ti(a, dt):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(dev)

    def time_events(fn, reps, warm=3):
        """Average duration (ms) of fn over `reps` back-to-back calls, HIP events on the launch stream."""
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    # ------------------------------------------------------------------------------------------------
    # the step's batch: 8B-shaped shard at P=8
    # ------------------------------------------------------------------------------------------------
    P, H, H_kv, D = 8, 32, 8, 128
    case = W.config2_attn()
    hq_l, hkv_l = case.hq_l, case.hkv_l
    n = case.total_q
    T = n // P
    log(f"[bench] step batch: {case.name}: {case.num_seqs} x {int(case.q_lens[0])} tokens, {hq_l}q/{hkv_l}kv heads, D={D}, "
        f"{case.num_blocks} cache blocks; flops/step = {case.flops() / 1e9:.2f} GFLOP (prefill)")

    rng = np.random.Generator(np.random.PCG64(1002))
    qkv_local = B.to_device(W.f32_to_bf16_bits(rng.standard_normal((T, H + 2 * H_kv, D), dtype=np.float32)), "bf16", dev)
    send = torch.empty((P, T, hq_l + 2 * hkv_l, D), dtype=bf, device=dev)
    new = case.new_token_index
    recv1 = B.to_device(np.concatenate([case.q, case.k_ctx[new], case.v_ctx[new]], axis=1), "bf16", dev)  # after a2a #1
    q_v, k_v, v_v = recv1[:, :hq_l], recv1[:, hq_l:hq_l + hkv_l], recv1[:, hq_l + hkv_l:]
    slots = ti(case.slots[new], np.int64)
    cache = torch.zeros((case.num_blocks, hkv_l, 2, 16 * D), dtype=bf, device=dev)
    table, cu, sl = ti(case.block_table, np.int32), ti(case.cu_seqlens_q, np.int32), ti(case.ctx_lens, np.int32)
    max_q, max_ctx = int(case.q_lens.max()), int(case.ctx_lens.max())
    attn_o = torch.empty((n, hq_l, D), dtype=bf, device=dev)
    recv2 = B.to_device(W.f32_to_bf16_bits(rng.standard_normal((P, T, hq_l, D), dtype=np.float32)), "bf16", dev)  # after a2a #2
    out_seq = torch.empty((T, H, D), dtype=bf, device=dev)
    # the decode step that follows for the same sequences (context 4097 each)
    dcase = W.make_attn_case("cfg2_decode_step", 1003, "bf16", [(1, int(c) + 1) for c in case.ctx_lens], hq_l, hkv_l, D,
                             pool_factor=2.0)
    dnew = dcase.new_token_index
    drecv = B.to_device(np.concatenate([dcase.q, dcase.k_ctx[dnew], dcase.v_ctx[dnew]], axis=1), "bf16", dev)
    dq, dk, dv = drecv[:, :hq_l], drecv[:, hq_l:hq_l + hkv_l], drecv[:, hq_l + hkv_l:]
    dslots = ti(dcase.slots[dnew], np.int64)
    dcache = torch.zeros((dcase.num_blocks, hkv_l, 2, 16 * D), dtype=bf, device=dev)
    dslots_all = dcase.slots.copy()
    dslots_all[dnew] = -1
    B.kv_write(B.to_device(dcase.k_ctx, "bf16", dev), B.to_device(dcase.v_ctx, "bf16", dev), ti(dslots_all, np.int64), dcache)
    dtable, dsl = ti(dcase.block_table, np.int32), ti(dcase.ctx_lens, np.int32)
    dmax = int(dcase.ctx_lens.max())
    dout = torch.empty((dcase.num_seqs, hq_l, D), dtype=bf, device=dev)
    a_dec = B.attn_desc(dq, dcache, dtable, dcase.softmax_scale, dk, dout)
    dws = torch.empty(max(B.decode_workspace_bytes(dcase.num_seqs, dmax, a_dec), 16), dtype=torch.uint8, device=dev)
    a_pre = B.attn_desc(q_v, cache, table, case.softmax_scale, k_v, attn_o)
    pws = torch.empty(max(B.prefill_workspace_bytes(case.num_seqs, n, max_q, max_ctx, a_pre), 16), dtype=torch.uint8, device=dev)

    def do_pack():
        B.pack_seq2head(qkv_local, send, P, H, H_kv)

    def do_prefill():
        B.prefill(q_v, cache, table, cu, sl, max_q, max_ctx, attn_o, case.softmax_scale, k_new=k_v, v_new=v_v,
                  slot_mapping=slots, workspace=pws)

    def do_prefill_kernel_only():
        B.prefill(q_v, cache, table, cu, sl, max_q, max_ctx, attn_o, case.softmax_scale, workspace=pws)

    def do_unpack():
        B.unpack_head2seq(recv2, out_seq)

    def do_decode():
        B.decode(dq, dcache, dtable, dsl, dmax, dout, dcase.softmax_scale, k_new=dk, v_new=dv, slot_mapping=dslots,
                 workspace=dws)

    def step():
        do_pack()
        do_prefill()
        do_unpack()
        do_decode()

    # ---- the timed region: W warm-up steps, then exactly K steps between synchronisations -----------------
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    step_flops = case.flops() + dcase.flops()
    value = step_flops / (ms_per_step * 1e-3) / 1e12
    log(f"[bench] step: {ms_per_step:.4f} ms -> {value:.1f} TFLOP/s of attention")
    # the same step captured once into a HIP graph and replayed (how the paper's engine issues it, Sec. 3.4); reported
    # beside the eager figure, which stays the headline
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_per_step_graph = (time.perf_counter() - t0) * 1e3 / args.steps
    log(f"[bench] step replayed from a HIP graph: {ms_per_step_graph:.4f} ms -> "
        f"{step_flops / (ms_per_step_graph * 1e-3) / 1e12:.1f} TFLOP/s")

    # ---- per-phase HIP-event timings, same stream ------------------------------------------------------------
    reps = max(args.steps, 10)
    phases = {}
    e = 2
    pack_bytes = T * (H + 2 * H_kv) * D * e + P * T * (hq_l + 2 * hkv_l) * D * e
    unpack_bytes = 2 * T * H * D * e
    for name, fn, work, unit in [("pack_seq2head", do_pack, pack_bytes / 1e9, "GB/s"),
                                 ("prefill_with_kv_write", do_prefill, case.flops() / 1e12, "TFLOP/s"),
                                 ("prefill_kernel", do_prefill_kernel_only, case.flops() / 1e12, "TFLOP/s"),
                                 ("unpack_head2seq", do_unpack, unpack_bytes / 1e9, "GB/s"),
                                 ("decode_with_kv_write", do_decode, dcase.kv_bytes() / 1e9, "GB/s")]:
        ms = time_events(fn, reps)
        phases[name] = {"ms": round(ms, 5), "rate": round(work / (ms * 1e-3), 2), "unit": unit}
        log(f"[bench]   {name:24s} {ms * 1e3:9.1f} us  {phases[name]['rate']:10.1f} {unit}")
    pk_ms = phases["prefill_kernel"]["ms"]
    achieved = case.flops() / (pk_ms * 1e-3) / 1e12
    roofline = {"kernel": "prefill_kernel (bf16 MFMA causal prefill)", "bound": "mfma", "achieved": round(achieved, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": traffic.get("prefill_8b"), "flops_per_launch": case.flops(), "avg_launch_ms": round(pk_ms, 5)}

    result = {
        "metric": METRIC, "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-3.1-8B-shaped shard at P=8, bf16, 4q/1kv heads, head_dim 128, "
                               "4 x 4096-token causal prefill, paged KV (16-token blocks, seeded random block table); "
                               "step = pack + prefill(+KV write) + unpack + one decode step",
                   "flop_convention": "4*D per (query, visible key) pair per query head",
                   "step_flops": step_flops},
        "roofline": roofline,
        "ms_per_step_graph_replay": round(ms_per_step_graph, 5),
        "phases": phases,
    }

    # ---- the HBM-bound kernels and the 70B-shaped prefill on their own configurations ------------------------
    if not args.no_extras:
        # batch decode, 256 sequences (configs[3])
        c4 = W.config4_attn()
        cache4 = torch.zeros((c4.num_blocks, 1, 2, 16 * D), dtype=bf, device=dev)
        B.kv_write(B.to_device(c4.k_ctx, "bf16", dev), B.to_device(c4.v_ctx, "bf16", dev), ti(c4.slots, np.int64), cache4)
        q4 = B.to_device(c4.q, "bf16", dev)
        t4, s4 = ti(c4.block_table, np.int32), ti(c4.ctx_lens, np.int32)
        o4 = torch.empty_like(q4)
        m4 = int(c4.ctx_lens.max())
        a4 = B.attn_desc(q4, cache4, t4, c4.softmax_scale, None, o4)
        w4 = torch.empty(B.decode_workspace_bytes(c4.num_seqs, m4, a4), dtype=torch.uint8, device=dev)
        ms = time_events(lambda: B.decode(q4, cache4, t4, s4, m4, o4, c4.softmax_scale, workspace=w4), reps)
        gbps = c4.kv_bytes() / (ms * 1e-3) / 1e9
        result["decode_kv_read"] = {"workload": f"configs[3]: 256 decode sequences, contexts U[512,8192], realised sum "
                                                f"{int(c4.ctx_lens.sum())} tokens, 8q/1kv, D=128, bf16 paged KV",
                                    "kv_bytes": c4.kv_bytes(), "ms": round(ms, 5),
                                    "roofline": {"kernel": "decode_flat_kernel + combine_flat_kernel", "bound": "hbm",
                                                 "achieved": round(gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                                 "frac": round(gbps / PEAK_HBM_GBPS, 4), "traffic": traffic.get("decode_256seq")}}
        log(f"[bench] decode cfg4: {ms * 1e3:.1f} us, {gbps:.0f} GB/s of KV ({gbps / PEAK_HBM_GBPS:.1%} of HBM peak)")
        # K/V append of the whole batch's contexts (the cache fill above, timed): read K and V rows, write cache blocks
        k4d, v4d, sl4 = B.to_device(c4.k_ctx, "bf16", dev), B.to_device(c4.v_ctx, "bf16", dev), ti(c4.slots, np.int64)
        ms = time_events(lambda: B.kv_write(k4d, v4d, sl4, cache4), 10)
        kvw_bytes = 2 * c4.kv_bytes()
        gbps = kvw_bytes / (ms * 1e-3) / 1e9
        result["kv_write"] = {"workload": f"K/V of all {int(c4.ctx_lens.sum())} context tokens of the configs[3] batch appended in one "
                                          "call (1 KV head, D=128, bf16; blocks scattered over the pool)",
                              "bytes": kvw_bytes, "ms": round(ms, 5),
                              "roofline": {"kernel": "kv_write_block_kernel", "bound": "hbm", "achieved": round(gbps, 1),
                                           "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(gbps / PEAK_HBM_GBPS, 4),
                                           "traffic": None}}
        log(f"[bench] kv_write of the cfg4 contexts: {ms * 1e3:.1f} us, {gbps:.0f} GB/s read + written ({gbps / PEAK_HBM_GBPS:.1%} of HBM peak)")
        del k4d, v4d, sl4
        # the same batch over an FP8 E4M3 cache: half the bytes per token
        k_scale, v_scale = 0.05, 0.05
        cache4q = torch.zeros((c4.num_blocks, 1, 2, 16 * D), dtype=torch.uint8, device=dev)
        B.kv_write(B.to_device(c4.k_ctx, "bf16", dev), B.to_device(c4.v_ctx, "bf16", dev), ti(c4.slots, np.int64), cache4q,
                   k_scale, v_scale)
        ms = time_events(lambda: B.decode(q4, cache4q, t4, s4, m4, o4, c4.softmax_scale, workspace=w4, k_scale=k_scale,
                                          v_scale=v_scale), reps)
        gbps = c4.kv_bytes() / 2 / (ms * 1e-3) / 1e9
        result["decode_kv_read_fp8"] = {"workload": "configs[3] batch over an FP8 E4M3 KV cache (1 byte per element, "
                                                    "per-tensor K and V scales)",
                                        "kv_bytes": c4.kv_bytes() // 2, "ms": round(ms, 5),
                                        "roofline": {"kernel": "decode_flat_kernel<fp8> + combine_flat_kernel", "bound": "hbm",
                                                     "achieved": round(gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                                     "frac": round(gbps / PEAK_HBM_GBPS, 4),
                                                     "traffic": traffic.get("decode_256seq_fp8")}}
        log(f"[bench] decode cfg4, FP8 cache: {ms * 1e3:.1f} us, {gbps:.0f} GB/s of KV ({gbps / PEAK_HBM_GBPS:.1%} of HBM peak)")
        del cache4, cache4q, w4
        # exchange of the 70B hidden state (configs[2])
        x3 = W.config3_xchg()
        copies = 3
        xin = [B.to_device(x3.x, "bf16", dev) for _ in range(copies)]
        xsend = [torch.empty((x3.P, x3.T_pad, x3.h // x3.P, D), dtype=bf, device=dev) for _ in range(copies)]
        xout = [torch.empty((x3.T, x3.h, D), dtype=bf, device=dev) for _ in range(copies)]
        it = [0]

        def pack3():
            i = it[0] = (it[0] + 1) % copies
            B.pack_seq2head(xin[i], xsend[i], x3.P, x3.h, 0)

        def unpack3():
            i = it[0] = (it[0] + 1) % copies
            B.unpack_head2seq(xsend[i], xout[i])

        for nm, fn in (("pack_seq2head", pack3), ("unpack_head2seq", unpack3)):
            ms = time_events(fn, reps)
            gbps = x3.bytes_moved() / (ms * 1e-3) / 1e9
            result[nm] = {"workload": "configs[2]: hidden [16384, 64 heads, 128] bf16 <-> 8 buffers, 3 rotating copies",
                          "bytes": x3.bytes_moved(), "ms": round(ms, 5),
                          "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                       "frac": round(gbps / PEAK_HBM_GBPS, 4), "traffic": traffic.get(nm + "_70b")}}
            log(f"[bench] {nm} cfg3: {ms * 1e3:.1f} us, {gbps:.0f} GB/s ({gbps / PEAK_HBM_GBPS:.1%} of HBM peak)")
        del xin, xsend, xout
        # the projections next to the two exchanges, fused with the pack / unpack (70B: d_model 8192, 64 + 2 x 8 heads)
        d_model, h3, hkv3 = 8192, 64, 8
        gen = torch.Generator(device=dev)
        gen.manual_seed(33)
        xe = torch.randn((x3.T, d_model), device=dev, generator=gen).to(bf)
        wq = (torch.randn(((h3 + 2 * hkv3) * D, d_model), device=dev, generator=gen) * 0.02).to(bf)
        wo = (torch.randn((d_model, h3 * D), device=dev, generator=gen) * 0.02).to(bf)
        send3 = torch.empty((x3.P, x3.T, h3 // x3.P + 2 * (hkv3 // x3.P), D), dtype=bf, device=dev)
        recv3 = torch.randn((x3.P, x3.T, h3 // x3.P, D), device=dev, generator=gen).to(bf)
        eo = torch.empty((x3.T, d_model), dtype=bf, device=dev)
        qkv_plain = torch.empty((x3.T, (h3 + 2 * hkv3) * D), dtype=bf, device=dev)
        att_plain = torch.empty((x3.T, h3 * D), dtype=bf, device=dev)

        def lib_qkv():   # the unfused route: the library's GEMM, then the pack kernel
            torch.matmul(xe, wq.t(), out=qkv_plain)
            B.pack_seq2head(qkv_plain.view(x3.T, h3 + 2 * hkv3, D), send3, x3.P, h3, hkv3)

        def lib_o():
            B.unpack_head2seq(recv3, att_plain.view(x3.T, h3, D))
            torch.matmul(att_plain, wo.t(), out=eo)

        for nm, fn, ref, fl in (("qkv_proj_pack", lambda: B.qkv_proj_pack(xe, wq, send3, x3.P, h3, hkv3), lib_qkv,
                                 2.0 * x3.T * d_model * (h3 + 2 * hkv3) * D),
                                ("unpack_o_proj", lambda: B.unpack_o_proj(recv3, wo, eo), lib_o, 2.0 * x3.T * d_model * h3 * D)):
            ms = time_events(fn, reps)
            ms_ref = time_events(ref, reps)
            tf = fl / (ms * 1e-3) / 1e12
            result[nm] = {"workload": f"configs[2] shard: {x3.T} tokens, d_model {d_model}, {h3} query + 2 x {hkv3} KV heads of 128, "
                                      f"{x3.P} exchange buffers, bf16, N(0,1) activations, N(0,0.02) weights",
                          "flops": fl, "ms": round(ms, 5), "library_gemm_and_separate_layout_kernel_ms": round(ms_ref, 5),
                          "roofline": {"kernel": "proj_gemm_kernel", "bound": "mfma", "achieved": round(tf, 2), "peak": PEAK_BF16_TFLOPS,
                                       "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4), "traffic": traffic.get(nm + "_70b")}}
            log(f"[bench] {nm} cfg3: {ms * 1e3:.1f} us, {tf:.1f} TFLOP/s ({tf / PEAK_BF16_TFLOPS:.1%} of bf16 MFMA peak); "
                f"library GEMM + separate layout kernel {ms_ref * 1e3:.1f} us")
        # the same two products with FP8 E4M3 operands: activations quantised per token on the fly, weights once
        PEAK_FP8_TFLOPS = 5000.0
        xq, xsc = torch.empty(xe.shape, dtype=torch.uint8, device=dev), torch.empty(x3.T, dtype=torch.float32, device=dev)
        wq8, wsc = torch.empty(wq.shape, dtype=torch.uint8, device=dev), torch.empty(wq.shape[0], dtype=torch.float32, device=dev)
        rq, rsc = torch.empty(recv3.shape, dtype=torch.uint8, device=dev), torch.empty(x3.T, dtype=torch.float32, device=dev)
        wo8, wosc = torch.empty(wo.shape, dtype=torch.uint8, device=dev), torch.empty(wo.shape[0], dtype=torch.float32, device=dev)
        B.quantize_rows_fp8(wq, wq8, wsc)
        B.quantize_rows_fp8(wo, wo8, wosc)
        B.quantize_rows_fp8(xe, xq, xsc)
        B.quantize_recv_fp8(recv3, rq, rsc)
        for nm, fn, qfn, fl in (("qkv_proj_pack_fp8", lambda: B.qkv_proj_pack_fp8(xq, xsc, wq8, wsc, send3, x3.P, h3, hkv3),
                                 lambda: B.quantize_rows_fp8(xe, xq, xsc), 2.0 * x3.T * d_model * (h3 + 2 * hkv3) * D),
                                ("unpack_o_proj_fp8", lambda: B.unpack_o_proj_fp8(rq, rsc, wo8, wosc, eo),
                                 lambda: B.quantize_recv_fp8(recv3, rq, rsc), 2.0 * x3.T * d_model * h3 * D)):
            ms = time_events(fn, reps)
            ms_q = time_events(qfn, reps)
            tf = fl / (ms * 1e-3) / 1e12
            q_bytes = 3.0 * x3.T * d_model if nm.startswith("qkv") else 3.0 * x3.T * h3 * D    # 2 bytes read, 1 written per element
            result[nm] = {"workload": result[nm[:-4]]["workload"] + "; operands as FP8 E4M3 codes with per-row scales, bf16 result",
                          "flops": fl, "ms": round(ms, 5),
                          "activation_quantiser": {"ms": round(ms_q, 5), "bytes": q_bytes,
                                                   "roofline": {"kernel": "quantize_rows_fp8_kernel", "bound": "hbm",
                                                                "achieved": round(q_bytes / (ms_q * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBPS,
                                                                "unit": "GB/s", "frac": round(q_bytes / (ms_q * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                                                                "traffic": None}},
                          "roofline": {"kernel": "proj_gemm_kernel<fp8>", "bound": "mfma", "achieved": round(tf, 2), "peak": PEAK_FP8_TFLOPS,
                                       "unit": "TFLOP/s", "frac": round(tf / PEAK_FP8_TFLOPS, 4), "traffic": traffic.get(nm + "_70b")}}
            log(f"[bench] {nm} cfg3: {ms * 1e3:.1f} us, {tf:.1f} TFLOP/s ({tf / PEAK_FP8_TFLOPS:.1%} of the fp8 MFMA peak); "
                f"quantising the activations {ms_q * 1e3:.1f} us ({q_bytes / (ms_q * 1e-3) / 1e9:.0f} GB/s)")
        del xe, wq, wo, send3, recv3, eo, qkv_plain, att_plain, xq, xsc, wq8, wsc, rq, rsc, wo8, wosc
        # 70B-shaped prefill (configs[2])
        c3 = W.config3_attn()
        cache3 = torch.zeros((c3.num_blocks, 1, 2, 16 * D), dtype=bf, device=dev)
        B.kv_write(B.to_device(c3.k_ctx, "bf16", dev), B.to_device(c3.v_ctx, "bf16", dev), ti(c3.slots, np.int64), cache3)
        q3 = B.to_device(c3.q, "bf16", dev)
        t3, cu3, s3 = ti(c3.block_table, np.int32), ti(c3.cu_seqlens_q, np.int32), ti(c3.ctx_lens, np.int32)
        o3 = torch.empty_like(q3)
        ms = time_events(lambda: B.prefill(q3, cache3, t3, cu3, s3, c3.total_q, c3.total_q, o3, c3.softmax_scale), reps)
        tf = c3.flops() / (ms * 1e-3) / 1e12
        result["prefill_70b"] = {"workload": "configs[2]: 8q/1kv, D=128, one 16384-token causal prefill", "flops": c3.flops(),
                                 "ms": round(ms, 5),
                                 "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": PEAK_BF16_TFLOPS,
                                              "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4),
                                              "traffic": traffic.get("prefill_70b")}}
        log(f"[bench] prefill cfg3: {ms * 1e3:.1f} us, {tf:.1f} TFLOP/s ({tf / PEAK_BF16_TFLOPS:.1%} of bf16 MFMA peak)")
        del cache3
        # mixed long-context step (configs[4]): one 2048-token chunk on a 131072-token cached context, then 64 decode
        # sequences, one shared block pool; both calls also write their new tokens' K/V
        c5, n_pre = W.config5_attn()
        pre5, dec5 = W.sub_case(c5, range(n_pre)), W.sub_case(c5, range(n_pre, c5.num_seqs))
        cache5 = torch.zeros((c5.num_blocks, 1, 2, 16 * D), dtype=bf, device=dev)
        cached_slots = c5.slots.copy()
        cached_slots[c5.new_token_index] = -1
        B.kv_write(B.to_device(c5.k_ctx, "bf16", dev), B.to_device(c5.v_ctx, "bf16", dev), ti(cached_slots, np.int64), cache5)

        def dev_case(c):
            nw = c.new_token_index
            return dict(q=B.to_device(c.q, "bf16", dev), k=B.to_device(c.k_ctx[nw], "bf16", dev),
                        v=B.to_device(c.v_ctx[nw], "bf16", dev), slots=ti(c.slots[nw], np.int64),
                        table=ti(c.block_table, np.int32), cu=ti(c.cu_seqlens_q, np.int32), sl=ti(c.ctx_lens, np.int32),
                        max_q=int(c.q_lens.max()), max_ctx=int(c.ctx_lens.max()))

        p5, d5 = dev_case(pre5), dev_case(dec5)
        p5["out"], d5["out"] = torch.empty_like(p5["q"]), torch.empty_like(d5["q"])
        ap5 = B.attn_desc(p5["q"], cache5, p5["table"], c5.softmax_scale, p5["k"], p5["out"])
        ad5 = B.attn_desc(d5["q"], cache5, d5["table"], c5.softmax_scale, d5["k"], d5["out"])
        wp5 = torch.empty(max(B.prefill_workspace_bytes(pre5.num_seqs, pre5.total_q, p5["max_q"], p5["max_ctx"], ap5), 16),
                          dtype=torch.uint8, device=dev)
        wd5 = torch.empty(max(B.decode_workspace_bytes(dec5.num_seqs, d5["max_ctx"], ad5), 16), dtype=torch.uint8, device=dev)

        def chunk5():
            B.prefill(p5["q"], cache5, p5["table"], p5["cu"], p5["sl"], p5["max_q"], p5["max_ctx"], p5["out"], c5.softmax_scale,
                      k_new=p5["k"], v_new=p5["v"], slot_mapping=p5["slots"], workspace=wp5)

        def decode5():
            B.decode(d5["q"], cache5, d5["table"], d5["sl"], d5["max_ctx"], d5["out"], c5.softmax_scale, k_new=d5["k"],
                     v_new=d5["v"], slot_mapping=d5["slots"], workspace=wd5)

        def both5():
            chunk5()
            decode5()

        # the same step as one unified batch through shiftattn_mixed (one K/V write for all rows)
        nw5 = c5.new_token_index
        u5 = dict(q=B.to_device(c5.q, "bf16", dev), k=B.to_device(c5.k_ctx[nw5], "bf16", dev),
                  v=B.to_device(c5.v_ctx[nw5], "bf16", dev), slots=ti(c5.slots[nw5], np.int64),
                  table=ti(c5.block_table, np.int32), cu=ti(c5.cu_seqlens_q[:n_pre + 1], np.int32), sl=ti(c5.ctx_lens, np.int32))
        u5["out"] = torch.empty_like(u5["q"])
        au5 = B.attn_desc(u5["q"], cache5, u5["table"], c5.softmax_scale, u5["k"], u5["out"])
        wu5 = torch.empty(max(B.mixed_workspace_bytes(n_pre, pre5.total_q, p5["max_q"], p5["max_ctx"], dec5.num_seqs,
                                                      d5["max_ctx"], au5), 16), dtype=torch.uint8, device=dev)

        def mixed5():
            B.mixed(u5["q"], cache5, u5["table"], u5["cu"], u5["sl"], n_pre, p5["max_q"], p5["max_ctx"], d5["max_ctx"],
                    u5["out"], c5.softmax_scale, k_new=u5["k"], v_new=u5["v"], slot_mapping=u5["slots"], workspace=wu5)

        ms_a, ms_b, ms_ab = time_events(chunk5, reps), time_events(decode5, reps), time_events(both5, reps)
        ms_u = time_events(mixed5, reps)
        # the same unified step over an FP8 E4M3 cache (the chunk's context is widened into the workspace first)
        cache5q = torch.zeros((c5.num_blocks, 1, 2, 16 * D), dtype=torch.uint8, device=dev)
        B.kv_write(B.to_device(c5.k_ctx, "bf16", dev), B.to_device(c5.v_ctx, "bf16", dev), ti(cached_slots, np.int64), cache5q,
                   0.05, 0.05)
        au5q = B.attn_desc(u5["q"], cache5q, u5["table"], c5.softmax_scale, u5["k"], u5["out"], 0.05, 0.05)
        wu5q = torch.empty(max(B.mixed_workspace_bytes(n_pre, pre5.total_q, p5["max_q"], p5["max_ctx"], dec5.num_seqs,
                                                       d5["max_ctx"], au5q), 16), dtype=torch.uint8, device=dev)
        ms_uq = time_events(lambda: B.mixed(u5["q"], cache5q, u5["table"], u5["cu"], u5["sl"], n_pre, p5["max_q"], p5["max_ctx"],
                                            d5["max_ctx"], u5["out"], c5.softmax_scale, k_new=u5["k"], v_new=u5["v"],
                                            slot_mapping=u5["slots"], workspace=wu5q, k_scale=0.05, v_scale=0.05), reps)
        del cache5q, wu5q
        tf5 = pre5.flops() / (ms_a * 1e-3) / 1e12
        gb5 = dec5.kv_bytes() / (ms_b * 1e-3) / 1e9
        result["mixed_long_context"] = {
            "workload": "configs[4]: 8q/1kv, D=128, bf16; (a) 2048-token chunk continuing a 131072-token cached context; "
                        f"(b) 64 decode sequences, contexts U[1024,32768], realised sum {int(dec5.ctx_lens.sum())} tokens; "
                        "both with the K/V write of their new tokens",
            "chunked_prefill": {"flops": pre5.flops(), "ms": round(ms_a, 5),
                                "roofline": {"bound": "mfma", "achieved": round(tf5, 2), "peak": PEAK_BF16_TFLOPS,
                                             "unit": "TFLOP/s", "frac": round(tf5 / PEAK_BF16_TFLOPS, 4), "traffic": None}},
            "decode": {"kv_bytes": dec5.kv_bytes(), "ms": round(ms_b, 5),
                       "roofline": {"bound": "hbm", "achieved": round(gb5, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                    "frac": round(gb5 / PEAK_HBM_GBPS, 4), "traffic": None}},
            "back_to_back_ms": round(ms_ab, 5), "unified_call_ms": round(ms_u, 5),
            "unified_call_fp8_cache_ms": round(ms_uq, 5)}
        log(f"[bench] mixed cfg5: chunk {ms_a * 1e3:.1f} us ({tf5:.1f} TFLOP/s, {tf5 / PEAK_BF16_TFLOPS:.1%}), decode "
            f"{ms_b * 1e3:.1f} us ({gb5:.0f} GB/s, {gb5 / PEAK_HBM_GBPS:.1%}), back to back {ms_ab * 1e3:.1f} us, as one unified call {ms_u * 1e3:.1f} us, "
            f"the same over an FP8 cache {ms_uq * 1e3:.1f} us")
        del cache5, wp5, wd5, wu5

    # ---- what the chip attains on the two priced resources (context for the roofline fractions) -------------
    if not args.no_extras:
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        ops = B.to_device(W.f32_to_bf16_bits(rng.standard_normal((128, 8), dtype=np.float32)), "bf16", dev)
        flops = [0]

        def mfma_probe():
            flops[0] = B.ceiling_mfma_bf16(ops, sink, 2000)

        ms = time_events(mfma_probe, 10)
        mfma_tf = flops[0] / (ms * 1e-3) / 1e12
        big = torch.empty(3 << 30, dtype=torch.uint8, device=dev)
        big.fill_(1)
        nbytes = [0]

        def read_probe():
            nbytes[0] = B.ceiling_hbm_read(big, sink)

        ms = time_events(read_probe, 5)
        rd_gbps = nbytes[0] / (ms * 1e-3) / 1e9
        result["attainable"] = {
            "mfma_bf16_random_operands": {"value": round(mfma_tf, 1), "unit": "TFLOP/s",
                                          "note": "MFMA-only loop, 32x32x16 bf16, N(0,1) operands, two wavefronts per SIMD"},
            "hbm_streaming_read": {"value": round(rd_gbps, 1), "unit": "GB/s",
                                   "note": "3 GiB read once by 2048 wavefronts, 16 KiB per wavefront in flight"}}
        log(f"[bench] attainable: MFMA-only loop {mfma_tf:.0f} TFLOP/s, streaming read {rd_gbps:.0f} GB/s")
        del big

    if args.pmc_calibrate:
        # a plain copy of known size, far larger than the caches: 512 Mi bf16 elements (1 GiB) read, as many written
        src = torch.ones(512 << 20, dtype=bf, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1, out=dst)
        torch.cuda.synchronize()
        log(f"[bench] calibration copy: {src.numel() * 2} bytes read and written per launch of torch's elementwise kernel")
        del src, dst

    # ---- CPU oracle on a bounded sample of the step's batch --------------------------------------------------
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        rows = np.arange(0, n, dtype=np.int64)                         # the whole prefill batch of the step
        ocache = O.cache_for_case(case)
        t0 = time.perf_counter()
        want = O.attention_case(case, ocache, rows)
        dt = time.perf_counter() - t0
        pos = np.concatenate([case.ctx_lens[s] - case.q_lens[s] + np.arange(case.q_lens[s]) for s in range(case.num_seqs)])
        sample_flops = 4 * D * hq_l * int((pos[rows] + 1).sum())
        do_prefill()
        torch.cuda.synchronize()
        got = W.to_f64(B.to_host(attn_o)[rows], "bf16")
        err = np.abs(got - want)
        result["cpu_baseline"] = {"value": round(sample_flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": O.num_threads(),
                                  "kind": "oracle", "seconds": round(dt, 2),
                                  "sample": f"fp64 oracle on every query token and head of the step's prefill batch "
                                            f"({sample_flops / 1e9:.1f} of {case.flops() / 1e9:.1f} GFLOP)"}
        result["parity_on_sample"] = {"max_abs_err": float(err.max()), "mean_abs_err": float(err.mean())}
        log(f"[bench] oracle: {dt:.1f} s on {O.num_threads()} threads, {sample_flops / dt / 1e9:.2f} GFLOP/s; "
            f"GPU vs oracle max|err|={err.max():.2e} mean|err|={err.mean():.2e}")

    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
