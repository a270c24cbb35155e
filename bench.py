#!/usr/bin/env python3
"""Benchmark of one GPU's share of a Shift-Parallelism attention layer on MI355X.

A "step" is one pass of the whole hot path over one synthetic batch, with every input already in HBM.  The batch
is the mixed long-context step of the 70B-shaped shard at P=8 (benchmark configs[4], the largest configuration
that is one GPU's work): one 2048-token chunk continuing a 131072-token cached context plus 64 decode sequences
with contexts uniform in [1024, 32768], 8 query heads / 1 KV head, head_dim 128, bf16, 16-token cache blocks in one
shared, randomly permuted pool.  The step is: send-side pack of this rank's fused QKV rows, the unified attention
call on chunk rows + decode rows (shiftattn_mixed: K/V append of all new tokens, chunked causal prefill, paged
decode, merges of split partials), receive-side unpack.  The wire exchange between ranks is not part of the path:
the buffers it would deliver are staged in HBM beforehand.

One JSON line goes to stdout.  `value` is attention TFLOP/s of the whole step (4*D flops per (query, visible key)
pair per query head, masked pairs and softmax not counted, over the wall time of the step).  `roofline` prices the
dominant kernel (the chunk's prefill kernel) against the chip's dense bf16 MFMA peak from HIP-event timing of that
call alone; `decode_in_step` prices the step's decode part against HBM bandwidth.  `cpu_baseline` is the fp64 CPU
oracle timed on a stated row sample of the same batch.  Further objects report the other configurations (8B-shaped
prefill batch, 70B-shaped prefill, 256-sequence decode, small decode batches, the 70B exchange, K/V append, the
fused projections), each with its own roofline object and an oracle timing.  All timings are medians of
per-call HIP-event pairs on the launch stream unless stated.  HBM traffic from hardware counters is not measured in
this run: `traffic` repeats the figure of the profiled runs summarised in profiles/hbm_traffic.md when that table was
measured on exactly the kernel sources of this tree (it carries their hash), and is null otherwise.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense fp8 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E
SETTLE_MS = 30.0            # load applied before a timed region so that the chip's clock has settled (main(): settle)
METRIC = "prefill attn TFLOP/s + decode KV-read GB/s per MI355X (head shard, % roofline)"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def source_stamp() -> str:
    """Hash of the kernel sources the library is built from (names and bytes of csrc/*)."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2509_16495_amd", "csrc", "*"))):
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def counter_traffic() -> dict:
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE of two rocprofv3 --pmc runs, scaled by a copy of known size) by
    workload key, from profiles/hbm_traffic.md - used only if that table was measured on exactly these kernel sources
    (it carries their stamp); otherwise every `traffic` stays null."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.md")
    out = {}
    try:
        text = open(path).read()
    except OSError:
        return out
    if f"source stamp: `{source_stamp()}`" not in text:
        return out
    for line in text.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 4 and cells[2].isdigit() and cells[3].isdigit():
            out[cells[0]] = int(cells[2]) + int(cells[3])
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--settle-scale", type=float, default=1.0,
                    help="scales the load applied before every timed region (0: none; counter runs do not need it)")
    ap.add_argument("--no-extras", action="store_true", help="only the headline step")
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
    dev = "cuda:0"
    torch.cuda.set_device(0)
    B.init()
    bf = torch.bfloat16
    D = 128
    cpu = not args.no_cpu_baseline
    if cpu:
        from oracle import oracle as O
        O.build()

    def ti(a, dt):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(dev)

    def settle(fn, ms=SETTLE_MS):
        """Calls fn back to back for `ms` of wall time.  After idling, the chip runs a matrix-heavy kernel up to 25 % slower
        for its first 15-20 ms of load (the shader clock under the power limit settles over some tens of launches: a
        16384-token prefill launch takes 610 us right after a pause and 472 us from the 40th launch on); a serving
        engine runs in the settled state, so that is the state every figure here is taken in."""
        t0, calls = time.perf_counter(), 0
        while (time.perf_counter() - t0) * 1e3 < ms * args.settle_scale and calls < 256:   # (launch-bound kernels: 256 calls do)
            for _ in range(4):
                fn()
            calls += 4
            torch.cuda.synchronize()

    def time_events(fn, reps, warm=3):
        """Median duration (ms) of fn over `reps` calls, one HIP-event pair per call on the launch stream."""
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        settle(fn)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in ev:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        return float(np.median([e0.elapsed_time(e1) for e0, e1 in ev]))

    def time_in_graph(fn, inner=20, reps=10):
        """ms per call of fn when `inner` calls are captured into one HIP graph and the graph is replayed back to back."""
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for _ in range(inner):
                    fn()
            g.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (inner * reps)

    traffic_by_key = counter_traffic()

    def roof(kernel, bound, achieved, peak, unit, traffic_key=None, **extra):
        r = {"kernel": kernel, "bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": unit,
             "frac": round(achieved / peak, 4), "traffic": traffic_by_key.get(traffic_key)}
        r.update(extra)
        return r

    def oracle_attention(case, rows, label):
        """fp64 oracle on the given query rows of a case: seconds, flops of the sample, outputs."""
        ocache = O.cache_for_case(case)
        t0 = time.perf_counter()
        want = O.attention_case(case, ocache, rows)
        dt = time.perf_counter() - t0
        pos = np.concatenate([case.ctx_lens[s] - case.q_lens[s] + np.arange(case.q_lens[s]) for s in range(case.num_seqs)])
        fl = 4 * case.D * case.hq_l * int((pos[rows] + 1).sum())
        return dt, fl, want

    def sample_rows(case, step=16, edge=32):
        """Every `step`-th query token of every sequence plus all tokens of its first and last `edge`."""
        rows = []
        for s in range(case.num_seqs):
            a, b = int(case.cu_seqlens_q[s]), int(case.cu_seqlens_q[s + 1])
            rows += list(range(a, b, step)) + list(range(a, min(a + edge, b))) + list(range(max(a, b - edge), b))
        return np.unique(np.array(rows, dtype=np.int64))

    reps = max(args.steps, 10)
    # ------------------------------------------------------------------------------------------------
    # the step's batch: configs[4], mixed long-context step of the 70B-shaped shard at P=8
    # ------------------------------------------------------------------------------------------------
    P, H, H_kv = 8, 64, 8
    c5, n_pre = W.config5_attn()
    pre5, dec5 = W.sub_case(c5, range(n_pre)), W.sub_case(c5, range(n_pre, c5.num_seqs))
    hq_l, hkv_l = c5.hq_l, c5.hkv_l
    n = c5.total_q                      # 2048 chunk rows + 64 decode rows
    T = n // P
    assert T * P == n
    log(f"[bench] step batch: {c5.name}: chunk {int(pre5.q_lens[0])} tokens on {int(pre5.ctx_lens[0] - pre5.q_lens[0])} cached, "
        f"{dec5.num_seqs} decode sequences (sum of contexts {int(dec5.ctx_lens.sum())}), {hq_l}q/{hkv_l}kv heads, D={D}, "
        f"{c5.num_blocks} cache blocks; {pre5.flops() / 1e9:.1f} GFLOP (chunk) + {dec5.kv_bytes() / 1e6:.1f} MB of KV (decodes)")
    rng = np.random.Generator(np.random.PCG64(5005))
    qkv_local = B.to_device(W.f32_to_bf16_bits(rng.standard_normal((T, H + 2 * H_kv, D), dtype=np.float32)), "bf16", dev)
    send = torch.empty((P, T, hq_l + 2 * hkv_l, D), dtype=bf, device=dev)
    nw5 = c5.new_token_index
    recv1 = B.to_device(np.concatenate([c5.q, c5.k_ctx[nw5], c5.v_ctx[nw5]], axis=1), "bf16", dev)   # after all-to-all #1
    q_v, k_v, v_v = recv1[:, :hq_l], recv1[:, hq_l:hq_l + hkv_l], recv1[:, hq_l + hkv_l:]
    slots5 = ti(c5.slots[nw5], np.int64)
    cache5 = torch.zeros((c5.num_blocks, hkv_l, 2, 16 * D), dtype=bf, device=dev)
    cached_slots = c5.slots.copy()
    cached_slots[nw5] = -1
    B.kv_write(B.to_device(c5.k_ctx, "bf16", dev), B.to_device(c5.v_ctx, "bf16", dev), ti(cached_slots, np.int64), cache5)
    table5, cu5, sl5 = ti(c5.block_table, np.int32), ti(c5.cu_seqlens_q[:n_pre + 1], np.int32), ti(c5.ctx_lens, np.int32)
    max_q5, max_pre5, max_dec5 = int(pre5.q_lens.max()), int(pre5.ctx_lens.max()), int(dec5.ctx_lens.max())
    attn_o = torch.empty((n, hq_l, D), dtype=bf, device=dev)
    recv2 = B.to_device(W.f32_to_bf16_bits(rng.standard_normal((P, T, hq_l, D), dtype=np.float32)), "bf16", dev)   # after all-to-all #2
    out_seq = torch.empty((T, H, D), dtype=bf, device=dev)
    a5 = B.attn_desc(q_v, cache5, table5, c5.softmax_scale, k_v, attn_o)
    ws5 = torch.empty(max(B.mixed_workspace_bytes(n_pre, pre5.total_q, max_q5, max_pre5, dec5.num_seqs, max_dec5, a5), 16),
                      dtype=torch.uint8, device=dev)
    n_chunk = pre5.total_q

    def do_pack():
        B.pack_seq2head(qkv_local, send, P, H, H_kv)

    def do_mixed():
        B.mixed(q_v, cache5, table5, cu5, sl5, n_pre, max_q5, max_pre5, max_dec5, attn_o, c5.softmax_scale, k_new=k_v, v_new=v_v,
                slot_mapping=slots5, workspace=ws5)

    def do_unpack():
        B.unpack_head2seq(recv2, out_seq)

    def do_chunk_only():      # the chunk's attention alone, cache already written
        B.prefill(q_v[:n_chunk], cache5, table5[:n_pre], cu5, sl5[:n_pre], max_q5, max_pre5, attn_o[:n_chunk], c5.softmax_scale,
                  workspace=ws5)

    def step():
        do_pack()
        do_mixed()
        do_unpack()

    # ---- the first K steps after a pause (the chip's clock has not settled: see settle()) -----------------
    step()
    torch.cuda.synchronize()
    time.sleep(0.2)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_after_idle = (time.perf_counter() - t0) * 1e3 / args.steps
    # ---- the timed region: the settled state, W warm-up steps, then exactly K steps between synchronisations ---------
    settle(step, 3 * SETTLE_MS)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    step_flops = c5.flops()
    value = step_flops / (ms_per_step * 1e-3) / 1e12
    log(f"[bench] step: {ms_per_step:.4f} ms -> {value:.1f} TFLOP/s of attention (first {args.steps} steps after a pause: "
        f"{ms_per_step_after_idle:.4f} ms)")
    # the same step captured once into a HIP graph and replayed (how the paper's engine issues it, Sec. 3.4)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    settle(graph.replay)
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_per_step_graph = (time.perf_counter() - t0) * 1e3 / args.steps
    log(f"[bench] step replayed from a HIP graph: {ms_per_step_graph:.4f} ms")

    # ---- the same step as separate calls in the same order, one HIP-event pair around every part (medians) -----------
    # pack | K/V append of all 2112 new rows | chunk attention (prefill64_kernel + the merge of its key ranges) |
    # the 64 decodes (decode kernel + merge) | unpack: the kernels of the unified call, each between two events on the
    # launch stream, every part in the cache state the step leaves it in (the chunk's 68 MB of K/V do not survive the
    # decodes' 538 MB in the 256 MB cache in front of HBM; timed alone in a loop they would)
    e = 2
    pack_bytes = T * (H + 2 * H_kv) * D * e + P * T * (hq_l + 2 * hkv_l) * D * e
    unpack_bytes = 2 * T * H * D * e

    def do_append():
        B.kv_write(k_v, v_v, slots5, cache5)

    def do_decode_part():
        B.decode(q_v[n_chunk:], cache5, table5[n_pre:], sl5[n_pre:], max_dec5, attn_o[n_chunk:], c5.softmax_scale, workspace=ws5)

    parts = [("pack_seq2head", do_pack, pack_bytes / 1e9, "GB/s"),
             ("kv_write_of_the_new_rows", do_append, 2.0 * n * hkv_l * D * e * 2 / 1e9, "GB/s"),
             ("chunk_prefill", do_chunk_only, pre5.flops() / 1e12, "TFLOP/s"),
             ("decodes", do_decode_part, dec5.kv_bytes() / 1e9, "GB/s"),
             ("unpack_head2seq", do_unpack, unpack_bytes / 1e9, "GB/s")]
    def all_parts():
        for _, fn, _, _ in parts:
            fn()

    settle(all_parts)
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(len(parts) + 1)] for _ in range(reps)]
    for ev in marks:
        ev[0].record()
        for i, (_, fn, _, _) in enumerate(parts):
            fn()
            ev[i + 1].record()
    torch.cuda.synchronize()
    phases = {}
    for i, (name, _, work, unit) in enumerate(parts):
        ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for ev in marks]))
        phases[name] = {"ms": round(ms, 5), "rate": round(work / (ms * 1e-3), 2), "unit": unit}
        log(f"[bench]   {name:32s} {ms * 1e3:9.1f} us  {phases[name]['rate']:10.1f} {unit}")
    ms = float(np.median([ev[0].elapsed_time(ev[-1]) for ev in marks]))
    phases["all_parts_as_separate_calls"] = {"ms": round(ms, 5), "rate": round(step_flops / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s"}
    ms = time_events(do_mixed, reps)
    phases["unified_call_alone"] = {"ms": round(ms, 5), "rate": round(step_flops / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s"}
    # how the chip settles: the chunk's attention call, 200 launches in a row after a pause, medians of ten
    torch.cuda.synchronize()
    time.sleep(0.5)
    sev = [torch.cuda.Event(enable_timing=True) for _ in range(201)]
    sev[0].record()
    for i in range(200):
        do_chunk_only()
        sev[i + 1].record()
    torch.cuda.synchronize()
    s_us = [sev[i].elapsed_time(sev[i + 1]) * 1e3 for i in range(200)]
    settling = [round(float(np.median(s_us[i:i + 10])), 1) for i in range(0, 200, 10)]
    log("[bench] chunk attention call, us per launch after a 0.5 s pause (medians of 10 launches): " + " ".join(f"{v:.0f}" for v in settling))
    ck_ms = phases["chunk_prefill"]["ms"]
    achieved = pre5.flops() / (ck_ms * 1e-3) / 1e12
    roofline = roof("prefill64_kernel (bf16 MFMA chunked prefill, one 256-column tile per workgroup over 4 key ranges; the call's combine_splits_kernel, about 1.5 % of it, is "
                    "inside the timed interval)", "mfma", achieved, PEAK_BF16_TFLOPS, "TFLOP/s",
                    traffic_key="chunk_prefill_long_context", flops_per_launch=pre5.flops(), median_launch_ms=round(ck_ms, 5))
    dd_ms = phases["decodes"]["ms"]
    dd_gbps = dec5.kv_bytes() / (dd_ms * 1e-3) / 1e9
    # the chunk's attention with the opt-in switch that lets Q carry the softmax scale (one more rounding of Q to bf16; off
    # by default and in everything else this run measures)
    B.set_option(B.OPT_PREFILL_SCALED_Q, 1)
    try:
        sq_ms = time_events(do_chunk_only, reps)
    finally:
        B.set_option(B.OPT_PREFILL_SCALED_Q, 0)
    sq_tf = pre5.flops() / (sq_ms * 1e-3) / 1e12
    log(f"[bench] chunk attention alone: with SHIFTATTN_OPT_PREFILL_SCALED_Q {sq_ms * 1e3:.1f} us, {sq_tf:.1f} TFLOP/s ({sq_tf / PEAK_BF16_TFLOPS:.1%} of peak)")

    result = {
        "metric": METRIC, "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[4]: mixed long-context step, Llama-3.3-70B-shaped shard at P=8, bf16, 8q/1kv heads, head_dim 128: "
                               "one 2048-token chunk continuing a 131072-token cached context + 64 decode sequences with contexts "
                               "U[1024,32768], paged KV (16-token blocks, one seeded random pool); "
                               "step = pack + unified attention call (K/V append, chunked prefill, decode) + unpack",
                   "flop_convention": "4*D per (query, visible key) pair per query head",
                   "step_flops": step_flops, "decode_kv_bytes": dec5.kv_bytes()},
        "roofline": roofline,
        "decode_in_step": {"kv_bytes": dec5.kv_bytes(), "ms": round(dd_ms, 5),
                           "roofline": roof("decode_flat_kernel + combine_flat_kernel", "hbm", dd_gbps, PEAK_HBM_GBPS, "GB/s", traffic_key="decode_64_long_contexts")},
        "ms_per_step_graph_replay": round(ms_per_step_graph, 5),
        "chunk_prefill_with_scaled_q": {
            "ms": round(sq_ms, 5), "roofline": roof("prefill64_kernel, SHIFTATTN_OPT_PREFILL_SCALED_Q = 1", "mfma", sq_tf, PEAK_BF16_TFLOPS, "TFLOP/s"),
            "note": "opt-in, not the path the step above runs: Q is multiplied by the softmax scale per tile and rounded to bf16 again and the "
                    "softmax takes no reference, so the loop spends no instruction on scaling and shifting logits; outputs of magnitude "
                    "2 and more can then land one bf16 step from the correctly rounded value (beyond the 2e-2 bound in 2 of 40 random batches); timed alone in a loop (the chunk's K/V then stay "
                    "in the cache in front of HBM, which makes it 2-3 % faster than inside the step)"},
        "timing_state": {"settle_ms": SETTLE_MS * args.settle_scale, "ms_per_step_first_steps_after_a_pause": round(ms_per_step_after_idle, 5),
                         "note": "every timed region starts after settle_ms (3x for the step) of the same work back to back: the "
                                 "chip's clock under the power limit takes 15-20 ms of load to settle, and matrix-heavy kernels run "
                                 "up to 25 % slower until then; the figure for the first steps after a 0.2 s pause is given beside it",
                         "chunk_prefill_us_per_launch_after_a_pause_medians_of_10": settling},
        "phases": phases,
        "traffic_note": "HBM bytes per launch (FETCH_SIZE + WRITE_SIZE) from the profiled runs in profiles/hbm_traffic.md; null when "
                        "that table was not measured on this tree's kernel sources",
    }

    # ---- CPU oracle on a bounded sample of the step's batch ---------------------------------------------------
    if cpu:
        rows = np.concatenate([sample_rows(pre5, step=4), np.arange(n_chunk, n)])   # chunk sample + every decode row
        dt, fl, want = oracle_attention(c5, rows, "cfg5")
        do_mixed()
        torch.cuda.synchronize()
        got = W.to_f64(B.to_host(attn_o)[rows], "bf16")
        err = np.abs(got - want)
        result["cpu_baseline"] = {
            "value": round(fl / dt / 1e12, 6), "unit": "TFLOP/s", "cores": O.num_threads(), "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"fp64 oracle on every 4th chunk token plus the first and last 32, all heads, and on all 64 decode rows "
                      f"({fl / 1e9:.1f} of {step_flops / 1e9:.1f} GFLOP)",
            "full_step_seconds_extrapolated": round(dt * step_flops / fl, 1)}
        result["parity_on_sample"] = {"max_abs_err": float(err.max()), "mean_abs_err": float(err.mean())}
        log(f"[bench] oracle: {dt:.1f} s on {O.num_threads()} threads, {fl / dt / 1e9:.2f} GFLOP/s; "
            f"GPU vs oracle max|err|={err.max():.2e} mean|err|={err.mean():.2e}")
    del cache5, ws5, recv1, recv2, send, qkv_local

    def cpu_obj(seconds, work, unit, sample):
        return {"value": round(work / seconds, 6), "unit": unit, "cores": O.num_threads(), "kind": "oracle",
                "seconds": round(seconds, 2), "sample": sample}

    # ------------------------------------------------------------------------------------------------
    # the other configurations
    # ------------------------------------------------------------------------------------------------
    if not args.no_extras:
        # ---- configs[1]: 8B-shaped prefill batch, 4 x 4096 tokens ------------------------------------------------
        c2 = W.config2_attn()
        new = c2.new_token_index
        r2 = B.to_device(np.concatenate([c2.q, c2.k_ctx[new], c2.v_ctx[new]], axis=1), "bf16", dev)
        q2, k2, v2 = r2[:, :c2.hq_l], r2[:, c2.hq_l:c2.hq_l + c2.hkv_l], r2[:, c2.hq_l + c2.hkv_l:]
        cache2 = torch.zeros((c2.num_blocks, c2.hkv_l, 2, 16 * D), dtype=bf, device=dev)
        t2, cu2, s2, sl2 = ti(c2.block_table, np.int32), ti(c2.cu_seqlens_q, np.int32), ti(c2.ctx_lens, np.int32), ti(c2.slots[new], np.int64)
        o2 = torch.empty((c2.total_q, c2.hq_l, D), dtype=bf, device=dev)
        mq2, mc2 = int(c2.q_lens.max()), int(c2.ctx_lens.max())
        ms_w = time_events(lambda: B.prefill(q2, cache2, t2, cu2, s2, mq2, mc2, o2, c2.softmax_scale, k_new=k2, v_new=v2,
                                             slot_mapping=sl2), reps)
        ms_k = time_events(lambda: B.prefill(q2, cache2, t2, cu2, s2, mq2, mc2, o2, c2.softmax_scale), reps)
        tf = c2.flops() / (ms_k * 1e-3) / 1e12
        result["prefill_8b"] = {"workload": "configs[1]: 4q/1kv, D=128, 4 x 4096-token causal prefill, paged KV", "flops": c2.flops(),
                                "ms": round(ms_k, 5), "ms_with_kv_write": round(ms_w, 5),
                                "roofline": roof("prefill_kernel (128-column tiles)", "mfma", tf, PEAK_BF16_TFLOPS, "TFLOP/s", traffic_key="prefill_8b")}
        log(f"[bench] prefill cfg2: {ms_k * 1e3:.1f} us ({ms_w * 1e3:.1f} with K/V write), {tf:.1f} TFLOP/s ({tf / PEAK_BF16_TFLOPS:.1%})")
        if cpu:
            dt, fl, _ = oracle_attention(c2, np.arange(c2.total_q, dtype=np.int64), "cfg2")
            result["prefill_8b"]["cpu_baseline"] = cpu_obj(dt, fl / 1e12, "TFLOP/s", "every query token and head of the batch")
        del cache2, r2

        # ---- configs[3]: batch decode, 256 sequences -------------------------------------------------------------
        c4 = W.config4_attn()
        cache4 = torch.zeros((c4.num_blocks, 1, 2, 16 * D), dtype=bf, device=dev)
        k4d, v4d, sl4 = B.to_device(c4.k_ctx, "bf16", dev), B.to_device(c4.v_ctx, "bf16", dev), ti(c4.slots, np.int64)
        B.kv_write(k4d, v4d, sl4, cache4)
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
                                    "roofline": roof("decode_flat_kernel + combine_flat_kernel", "hbm", gbps, PEAK_HBM_GBPS, "GB/s", traffic_key="decode_256seq")}
        # the same call as a serving loop issues it: captured into a HIP graph (the gap between the kernel and its merge shrinks)
        ms_g = time_in_graph(lambda: B.decode(q4, cache4, t4, s4, m4, o4, c4.softmax_scale, workspace=w4), inner=10, reps=5)
        result["decode_kv_read"]["replayed_from_graph"] = {"ms": round(ms_g, 5), "GB/s": round(c4.kv_bytes() / (ms_g * 1e-3) / 1e9, 1),
                                                           "frac": round(c4.kv_bytes() / (ms_g * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)}
        log(f"[bench] decode cfg4: {ms * 1e3:.1f} us, {gbps:.0f} GB/s of KV ({gbps / PEAK_HBM_GBPS:.1%} of HBM peak); replayed from a graph {ms_g * 1e3:.1f} us")
        if cpu:
            sub = W.sub_case(c4, range(0, c4.num_seqs, 4))
            dt, fl, _ = oracle_attention(sub, np.arange(sub.total_q, dtype=np.int64), "cfg4")
            result["decode_kv_read"]["cpu_baseline"] = cpu_obj(dt, sub.kv_bytes() / 1e9, "GB/s", "every 4th sequence of the batch (64 of 256), all heads")
        # K/V append of the whole batch's contexts: read K and V rows, write cache blocks
        ms = time_events(lambda: B.kv_write(k4d, v4d, sl4, cache4), 10)
        kvw_bytes = 2 * c4.kv_bytes()
        gbps = kvw_bytes / (ms * 1e-3) / 1e9
        # what a plain copy of the same bytes attains on this chip (read + write stream, the shape of this kernel's traffic)
        cp_src, cp_dst = torch.empty(kvw_bytes // 2, dtype=torch.uint8, device=dev), torch.empty(kvw_bytes // 2, dtype=torch.uint8, device=dev)
        cp_src.fill_(1)
        ms_cp = time_events(lambda: B.copy_probe(cp_src, cp_dst), 10)
        del cp_src, cp_dst
        result["kv_write"] = {"workload": f"K/V of all {int(c4.ctx_lens.sum())} context tokens of the configs[3] batch appended in one "
                                          "call (1 KV head, D=128, bf16; blocks scattered over the pool)",
                              "bytes": kvw_bytes, "ms": round(ms, 5),
                              "roofline": roof("kv_write_block_kernel", "hbm", gbps, PEAK_HBM_GBPS, "GB/s", traffic_key="kv_write_256seq"),
                              "streaming_copy_of_the_same_bytes": {"ms": round(ms_cp, 5), "GB/s": round(kvw_bytes / (ms_cp * 1e-3) / 1e9, 1),
                                                                   "note": "this library's own read+write probe (16-byte non-temporal "
                                                                           "loads and stores, no index arithmetic)"}}
        log(f"[bench] kv_write of the cfg4 contexts: {ms * 1e3:.1f} us, {gbps:.0f} GB/s read + written ({gbps / PEAK_HBM_GBPS:.1%} of HBM peak); "
            f"a plain copy of the same bytes: {ms_cp * 1e3:.1f} us")
        if cpu:
            n_tok = 200000
            t0 = time.perf_counter()
            oc = O.new_cache(c4.num_blocks, 1, 16, D, "bf16")
            O.kv_write(oc, c4.k_ctx[:n_tok], c4.v_ctx[:n_tok], c4.slots[:n_tok], 16, "bf16")
            dt = time.perf_counter() - t0
            result["kv_write"]["cpu_baseline"] = cpu_obj(dt, n_tok * 2 * 2 * D * 2 / 1e9, "GB/s", f"the first {n_tok} context tokens of the batch")
            del oc
        del k4d, v4d, sl4
        # the same batch over an FP8 E4M3 cache: half the bytes per token
        k_scale, v_scale = 0.05, 0.05
        cache4q = torch.zeros((c4.num_blocks, 1, 2, 16 * D), dtype=torch.uint8, device=dev)
        B.kv_write(B.to_device(c4.k_ctx, "bf16", dev), B.to_device(c4.v_ctx, "bf16", dev), ti(c4.slots, np.int64), cache4q,
                   k_scale, v_scale)
        ms = time_events(lambda: B.decode(q4, cache4q, t4, s4, m4, o4, c4.softmax_scale, workspace=w4, k_scale=k_scale,
                                          v_scale=v_scale), reps)
        gbps = c4.kv_bytes() / 2 / (ms * 1e-3) / 1e9
        result["decode_kv_read_fp8"] = {"workload": "configs[3] batch over an FP8 E4M3 KV cache (1 byte per element, per-tensor K and V scales)",
                                        "kv_bytes": c4.kv_bytes() // 2, "ms": round(ms, 5),
                                        "roofline": roof("decode_flat_kernel<fp8> + combine_flat_kernel", "hbm", gbps, PEAK_HBM_GBPS, "GB/s", traffic_key="decode_256seq_fp8")}
        ms_g = time_in_graph(lambda: B.decode(q4, cache4q, t4, s4, m4, o4, c4.softmax_scale, workspace=w4, k_scale=k_scale,
                                              v_scale=v_scale), inner=10, reps=5)
        result["decode_kv_read_fp8"]["replayed_from_graph"] = {"ms": round(ms_g, 5), "GB/s": round(c4.kv_bytes() / 2 / (ms_g * 1e-3) / 1e9, 1),
                                                               "frac": round(c4.kv_bytes() / 2 / (ms_g * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)}
        log(f"[bench] decode cfg4, FP8 cache: {ms * 1e3:.1f} us, {gbps:.0f} GB/s of KV ({gbps / PEAK_HBM_GBPS:.1%} of HBM peak); replayed from a graph {ms_g * 1e3:.1f} us")
        if cpu:
            sub = W.sub_case(c4, range(0, c4.num_seqs, 8))
            t0 = time.perf_counter()
            O.attention_case(sub, O.cache_for_case(sub, fp8_scales=(k_scale, v_scale)), k_scale=k_scale, v_scale=v_scale)
            dt = time.perf_counter() - t0
            result["decode_kv_read_fp8"]["cpu_baseline"] = cpu_obj(dt, sub.kv_bytes() / 2 / 1e9, "GB/s",
                                                                   "every 8th sequence of the batch (32 of 256), all heads, cache build included")
        del cache4, cache4q, w4

        # ---- small decode batches (the shift configuration's regime, Algorithm 2: few tokens per step) ----------------
        small = {}
        for ctx_len in (4096, 32768):
            for nseq in (1, 4, 16, 64):
                cs = W.make_attn_case("small_decode", 700 + nseq, "bf16", [(1, ctx_len + 1)] * nseq, 8, 1, D, pool_factor=1.1)
                cch = torch.zeros((cs.num_blocks, 1, 2, 16 * D), dtype=bf, device=dev)
                sl_all = cs.slots.copy()
                sl_all[cs.new_token_index] = -1
                B.kv_write(B.to_device(cs.k_ctx, "bf16", dev), B.to_device(cs.v_ctx, "bf16", dev), ti(sl_all, np.int64), cch)
                fz = B.to_device(np.concatenate([cs.q, cs.k_ctx[cs.new_token_index], cs.v_ctx[cs.new_token_index]], axis=1), "bf16", dev)
                qs, ks, vs = fz[:, :8], fz[:, 8:9], fz[:, 9:]
                ts_, ss_, sls = ti(cs.block_table, np.int32), ti(cs.ctx_lens, np.int32), ti(cs.slots[cs.new_token_index], np.int64)
                os_ = torch.empty((nseq, 8, D), dtype=bf, device=dev)
                as_ = B.attn_desc(qs, cch, ts_, cs.softmax_scale, ks, os_)
                wss = torch.empty(B.decode_workspace_bytes(nseq, ctx_len + 1, as_), dtype=torch.uint8, device=dev)
                def step_small():
                    B.decode(qs, cch, ts_, ss_, ctx_len + 1, os_, cs.softmax_scale, k_new=ks, v_new=vs, slot_mapping=sls, workspace=wss)
                ms = time_events(step_small, reps)
                us_graph = time_in_graph(step_small) * 1e3
                small[f"{nseq}x{ctx_len + 1}"] = {"us": round(ms * 1e3, 2), "us_replayed_from_graph": round(us_graph, 2), "kv_bytes": cs.kv_bytes(),
                                                  "GB/s": round(cs.kv_bytes() / (us_graph * 1e-6) / 1e9, 1)}
                del cch, wss
        result["decode_small_batches"] = {"workload": "decode steps of 1 / 4 / 16 / 64 sequences at contexts 4097 and 32769 (8q/1kv, D=128, bf16), "
                                                      "each with its K/V append; us = HIP-event median around single calls, "
                                                      "us_replayed_from_graph = 20 steps captured into one HIP graph, replayed back to back (Sec. 3.4)",
                                          "bound": "latency below a few MB of KV, hbm above", "calls": small}
        log("[bench] small decode batches (us per call / per step of a replayed graph): " +
            ", ".join(f"{k}: {v['us']} / {v['us_replayed_from_graph']}" for k, v in small.items()))

        # ---- configs[2]: exchange of the 70B hidden state ----------------------------------------------------------
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
                          "roofline": roof(nm + "_kernel", "hbm", gbps, PEAK_HBM_GBPS, "GB/s", traffic_key=nm + "_70b")}
            log(f"[bench] {nm} cfg3: {ms * 1e3:.1f} us, {gbps:.0f} GB/s ({gbps / PEAK_HBM_GBPS:.1%} of HBM peak)")
        if cpu:
            t0 = time.perf_counter()
            sp = O.pack_seq2head(x3.x, x3.P, x3.h, 0, x3.T_pad, "bf16")
            dt = time.perf_counter() - t0
            result["pack_seq2head"]["cpu_baseline"] = cpu_obj(dt, x3.bytes_moved() / 1e9, "GB/s", "the whole hidden state")
            t0 = time.perf_counter()
            O.unpack_head2seq(sp, x3.T, "bf16")
            dt = time.perf_counter() - t0
            result["unpack_head2seq"]["cpu_baseline"] = cpu_obj(dt, x3.bytes_moved() / 1e9, "GB/s", "the whole hidden state")
            del sp
        del xin, xsend, xout

        # ---- the projections next to the two exchanges, fused with the pack / unpack (70B: d_model 8192) ------------
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
                          "roofline": roof("proj_gemm_kernel", "mfma", tf, PEAK_BF16_TFLOPS, "TFLOP/s", traffic_key=nm + "_70b")}
            log(f"[bench] {nm} cfg3: {ms * 1e3:.1f} us, {tf:.1f} TFLOP/s ({tf / PEAK_BF16_TFLOPS:.1%} of bf16 MFMA peak); "
                f"library GEMM + separate layout kernel {ms_ref * 1e3:.1f} us")
        n_cpu_rows = 2048   # token rows of these products that the oracle is timed on
        if cpu:
            x_h, wq_h, wo_h = B.to_host(xe[:n_cpu_rows]), B.to_host(wq), B.to_host(wo)
            recv_h = B.to_host(recv3[:, :n_cpu_rows].contiguous())
            t0 = time.perf_counter()
            O.qkv_proj_pack(x_h, wq_h, x3.P, h3, hkv3, D, n_cpu_rows, "bf16")
            dt = time.perf_counter() - t0
            result["qkv_proj_pack"]["cpu_baseline"] = cpu_obj(dt, 2.0 * n_cpu_rows * d_model * wq.shape[0] / 1e12, "TFLOP/s",
                                                              f"the first {n_cpu_rows} token rows, all features")
            t0 = time.perf_counter()
            O.unpack_o_proj(recv_h, wo_h, n_cpu_rows, "bf16")
            dt = time.perf_counter() - t0
            result["unpack_o_proj"]["cpu_baseline"] = cpu_obj(dt, 2.0 * n_cpu_rows * d_model * h3 * D / 1e12, "TFLOP/s",
                                                              f"the first {n_cpu_rows} token rows, all features")
            del x_h, recv_h
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
                                                   "roofline": roof("quantize_rows_fp8_kernel", "hbm", q_bytes / (ms_q * 1e-3) / 1e9,
                                                                    PEAK_HBM_GBPS, "GB/s")},
                          "roofline": roof("proj_gemm_kernel<fp8>", "mfma", tf, PEAK_FP8_TFLOPS, "TFLOP/s", traffic_key=nm + "_70b")}
            log(f"[bench] {nm} cfg3: {ms * 1e3:.1f} us, {tf:.1f} TFLOP/s ({tf / PEAK_FP8_TFLOPS:.1%} of the fp8 MFMA peak); "
                f"quantising the activations {ms_q * 1e3:.1f} us ({q_bytes / (ms_q * 1e-3) / 1e9:.0f} GB/s)")
        if cpu:
            xq_h, xsc_h = B.to_host(xq[:n_cpu_rows]), B.to_host(xsc[:n_cpu_rows])
            rq_h, rsc_h = B.to_host(rq[:, :n_cpu_rows].contiguous()), B.to_host(rsc[:n_cpu_rows])
            wq8_h, wsc_h, wo8_h, wosc_h = B.to_host(wq8), B.to_host(wsc), B.to_host(wo8), B.to_host(wosc)
            t0 = time.perf_counter()
            O.qkv_proj_pack_fp8(xq_h, xsc_h, wq8_h, wsc_h, x3.P, h3, hkv3, D, n_cpu_rows)
            dt = time.perf_counter() - t0
            result["qkv_proj_pack_fp8"]["cpu_baseline"] = cpu_obj(dt, 2.0 * n_cpu_rows * d_model * wq.shape[0] / 1e12, "TFLOP/s",
                                                                  f"the first {n_cpu_rows} token rows, all features")
            t0 = time.perf_counter()
            O.unpack_o_proj_fp8(rq_h, rsc_h, wo8_h, wosc_h, n_cpu_rows)
            dt = time.perf_counter() - t0
            result["unpack_o_proj_fp8"]["cpu_baseline"] = cpu_obj(dt, 2.0 * n_cpu_rows * d_model * h3 * D / 1e12, "TFLOP/s",
                                                                  f"the first {n_cpu_rows} token rows, all features")
            del xq_h, rq_h, wq8_h, wo8_h

        # ---- the same projections at the token counts of a decode step (Algorithm 2: below the threshold) ---------
        # three copies of each weight matrix in rotation (504 / 403 MB), so that no pass is served from the 256 MB cache in
        # front of HBM; every figure is the time per call of 12 calls captured in one HIP graph and replayed
        wq_rot = [wq] + [(torch.randn(wq.shape, device=dev, generator=gen) * 0.02).to(bf) for _ in range(2)]
        wo_rot = [wo] + [(torch.randn(wo.shape, device=dev, generator=gen) * 0.02).to(bf) for _ in range(2)]
        small_proj = {}
        for Ts in (1, 8, 16, 32, 64, 256):
            xs_ = torch.randn((Ts, d_model), device=dev, generator=gen).to(bf)
            snd = torch.empty((x3.P, Ts, h3 // x3.P + 2 * (hkv3 // x3.P), D), dtype=bf, device=dev)
            rcv = torch.randn((x3.P, Ts, h3 // x3.P, D), device=dev, generator=gen).to(bf)
            eo_s = torch.empty((Ts, d_model), dtype=bf, device=dev)
            plain_q = torch.empty((Ts, (h3 + 2 * hkv3) * D), dtype=bf, device=dev)
            plain_a = torch.empty((Ts, h3 * D), dtype=bf, device=dev)
            ws_q = torch.empty(max(B.proj_workspace_bytes(Ts, wq.shape[0], d_model), 16), dtype=torch.uint8, device=dev)
            ws_o = torch.empty(max(B.proj_workspace_bytes(Ts, d_model, h3 * D), 16), dtype=torch.uint8, device=dev)
            turn = [0]

            def nxt(lst):
                turn[0] = (turn[0] + 1) % 3
                return lst[turn[0]]

            def lib_q_small():
                torch.matmul(xs_, nxt(wq_rot).t(), out=plain_q)
                B.pack_seq2head(plain_q.view(Ts, h3 + 2 * hkv3, D), snd, x3.P, h3, hkv3)

            def lib_o_small():
                B.unpack_head2seq(rcv, plain_a.view(Ts, h3, D))
                torch.matmul(plain_a, nxt(wo_rot).t(), out=eo_s)

            row = {}
            for nm, fn, ref, wbytes in (("qkv_proj_pack", lambda: B.qkv_proj_pack(xs_, nxt(wq_rot), snd, x3.P, h3, hkv3, workspace=ws_q),
                                         lib_q_small, wq.numel() * 2),
                                        ("unpack_o_proj", lambda: B.unpack_o_proj(rcv, nxt(wo_rot), eo_s, workspace=ws_o),
                                         lib_o_small, wo.numel() * 2)):
                us, us_ref = time_in_graph(fn, inner=12) * 1e3, time_in_graph(ref, inner=12) * 1e3
                gbps = wbytes / (us * 1e-6) / 1e9
                row[nm] = {"us": round(us, 2), "library_gemm_and_separate_layout_kernel_us": round(us_ref, 2),
                           "weight_bytes": wbytes, "us_to_stream_the_weights_at_peak": round(wbytes / PEAK_HBM_GBPS / 1e3, 2),
                           "roofline": roof("proj_stream_kernel" if Ts <= 64 else "proj_gemm_kernel<bf16>", "hbm", gbps, PEAK_HBM_GBPS, "GB/s", traffic_key=f"{nm}_T{Ts}")}
            small_proj[f"T={Ts}"] = row
            if cpu and Ts == 16:
                t0 = time.perf_counter()
                O.qkv_proj_pack(B.to_host(xs_), B.to_host(wq), x3.P, h3, hkv3, D, Ts, "bf16")
                dt = time.perf_counter() - t0
                small_proj["cpu_baseline"] = cpu_obj(dt, 2.0 * Ts * d_model * wq.shape[0] / 1e9, "GFLOP/s", "qkv_proj_pack of the 16-token call, whole")
            del xs_, snd, rcv, eo_s, plain_q, plain_a, ws_q, ws_o
        # the same over FP8 operands (four weight copies in rotation: 336 / 268 MB)
        wq8_rot = [wq8] + [wq8.clone() for _ in range(3)]
        wo8_rot = [wo8] + [wo8.clone() for _ in range(3)]
        small_fp8 = {}
        for Ts in (1, 8, 16, 32, 64, 256):
            xq_s, xsc_s = xq[:Ts].contiguous(), xsc[:Ts].contiguous()
            rq_s, rsc_s = rq[:, :Ts].contiguous(), rsc[:Ts].contiguous()
            snd = torch.empty((x3.P, Ts, h3 // x3.P + 2 * (hkv3 // x3.P), D), dtype=bf, device=dev)
            eo_s = torch.empty((Ts, d_model), dtype=bf, device=dev)
            ws_q = torch.empty(max(B.proj_workspace_bytes(Ts, wq.shape[0], d_model, fp8=True), 16), dtype=torch.uint8, device=dev)
            ws_o = torch.empty(max(B.proj_workspace_bytes(Ts, d_model, h3 * D, fp8=True), 16), dtype=torch.uint8, device=dev)
            turn = [0]

            def nxt4(lst):
                turn[0] = (turn[0] + 1) % 4
                return lst[turn[0]]

            row = {}
            for nm, fn, wbytes in (("qkv_proj_pack_fp8", lambda: B.qkv_proj_pack_fp8(xq_s, xsc_s, nxt4(wq8_rot), wsc, snd, x3.P, h3, hkv3, workspace=ws_q),
                                    wq8.numel()),
                                   ("unpack_o_proj_fp8", lambda: B.unpack_o_proj_fp8(rq_s, rsc_s, nxt4(wo8_rot), wosc, eo_s, workspace=ws_o),
                                    wo8.numel())):
                us = time_in_graph(fn, inner=12) * 1e3
                row[nm] = {"us": round(us, 2), "weight_bytes": wbytes, "us_to_stream_the_weights_at_peak": round(wbytes / PEAK_HBM_GBPS / 1e3, 2),
                           "roofline": roof("proj_stream_kernel<fp8>" if Ts <= 64 else "proj_gemm_kernel<fp8> (k split over workgroups) + proj_stream_finish_kernel", "hbm",
                                            wbytes / (us * 1e-6) / 1e9, PEAK_HBM_GBPS, "GB/s")}
            small_fp8[f"T={Ts}"] = row
            del snd, eo_s, ws_q, ws_o
        small_proj["fp8_operands"] = small_fp8
        log("[bench] the same over FP8 operands, us: " +
            ", ".join(f"{k}: qkv {v['qkv_proj_pack_fp8']['us']} o {v['unpack_o_proj_fp8']['us']}" for k, v in small_fp8.items()))
        del wq8_rot, wo8_rot
        result["decode_sized_projections"] = {
            "workload": f"the configs[2] shard's projections (d_model {d_model}, {h3} query + 2 x {hkv3} KV heads of 128, {x3.P} exchange buffers, bf16) "
                        "at 1 .. 256 token rows; one pass over the weights bounds them",
            "calls": small_proj}
        log("[bench] projections at decode-sized token counts, us (ours / library GEMM + layout kernel): " +
            ", ".join(f"{k}: qkv {v['qkv_proj_pack']['us']}/{v['qkv_proj_pack']['library_gemm_and_separate_layout_kernel_us']} "
                      f"o {v['unpack_o_proj']['us']}/{v['unpack_o_proj']['library_gemm_and_separate_layout_kernel_us']}"
                      for k, v in small_proj.items() if k.startswith("T=")))
        del wq_rot, wo_rot
        del xe, wq, wo, send3, recv3, eo, qkv_plain, att_plain, xq, xsc, wq8, wsc, rq, rsc, wo8, wosc

        # ---- configs[2]: 70B-shaped prefill; and the same length with 5 query heads per KV head (Table 4, Llama-17B-16E at P=8)
        for key, case, label in (("prefill_70b", W.config3_attn(), "configs[2]: 8q/1kv, D=128, one 16384-token causal prefill"),
                                 ("prefill_5q_per_kv", W.make_attn_case("g5_16k", 35, "bf16", [(16384, 16384)], 5, 1, D),
                                  "40q/8kv model on 8 ranks: 5q/1kv, D=128, one 16384-token causal prefill (not a BASELINE config)"),
                                 ("prefill_unequal_prompts", W.make_attn_case("mix3", 36, "bf16", [(12000, 12000), (7000, 7000), (3000, 3000)], 8, 1, D),
                                  "8q/1kv, D=128, three prompts of 12000 + 7000 + 3000 tokens prefilled in one batch (not a BASELINE config)")):
            cch = torch.zeros((case.num_blocks, 1, 2, 16 * D), dtype=bf, device=dev)
            B.kv_write(B.to_device(case.k_ctx, "bf16", dev), B.to_device(case.v_ctx, "bf16", dev), ti(case.slots, np.int64), cch)
            q3 = B.to_device(case.q, "bf16", dev)
            t3, cu3, s3 = ti(case.block_table, np.int32), ti(case.cu_seqlens_q, np.int32), ti(case.ctx_lens, np.int32)
            o3 = torch.empty_like(q3)
            mq3, mc3 = int(case.q_lens.max()), int(case.ctx_lens.max())
            ms = time_events(lambda: B.prefill(q3, cch, t3, cu3, s3, mq3, mc3, o3, case.softmax_scale), reps)
            tf = case.flops() / (ms * 1e-3) / 1e12
            kname = ("prefill64_kernel (256-column tiles in pairs)" if key == "prefill_70b" else
                     "prefill64_kernel (256-column tiles one per workgroup, heaviest first" + (", 2 key ranges)" if key == "prefill_5q_per_kv" else ")"))
            result[key] = {"workload": label, "flops": case.flops(), "ms": round(ms, 5),
                           "roofline": roof(kname, "mfma", tf, PEAK_BF16_TFLOPS, "TFLOP/s", traffic_key=key)}
            log(f"[bench] {key}: {ms * 1e3:.1f} us, {tf:.1f} TFLOP/s ({tf / PEAK_BF16_TFLOPS:.1%} of bf16 MFMA peak)")
            if cpu:
                rows = sample_rows(case, step=256, edge=32)
                dt, fl, want = oracle_attention(case, rows, key)
                err = np.abs(W.to_f64(B.to_host(o3)[rows], "bf16") - want)
                result[key]["cpu_baseline"] = cpu_obj(dt, fl / 1e12, "TFLOP/s", "every 256th query token plus the first and last 32, all heads")
                result[key]["parity_on_sample"] = {"max_abs_err": float(err.max()), "mean_abs_err": float(err.mean())}
            del cch

        # ---- what the chip attains on the two priced resources (context for the roofline fractions) -------------
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        ops = B.to_device(W.f32_to_bf16_bits(rng.standard_normal((128, 8), dtype=np.float32)), "bf16", dev)
        flops = [0]

        def mfma_probe():
            flops[0] = B.ceiling_mfma_bf16(ops, sink, 2000)

        ms = time_events(mfma_probe, 10)
        mfma_tf = flops[0] / (ms * 1e-3) / 1e12
        ops16 = B.to_device(W.f32_to_bf16_bits(rng.standard_normal((1024, 8), dtype=np.float32)), "bf16", dev)

        def mfma_fresh_probe():
            flops[0] = B.ceiling_mfma_bf16_fresh(ops16, sink, 1000)

        ms = time_events(mfma_fresh_probe, 10)
        mfma_fresh_tf = flops[0] / (ms * 1e-3) / 1e12
        big = torch.empty(3 << 30, dtype=torch.uint8, device=dev)
        big.fill_(1)
        nbytes = [0]

        def read_probe():
            nbytes[0] = B.ceiling_hbm_read(big, sink)

        ms = time_events(read_probe, 5)
        rd_gbps = nbytes[0] / (ms * 1e-3) / 1e9
        result["attainable"] = {
            "mfma_bf16_random_operands": {"value": round(mfma_tf, 1), "unit": "TFLOP/s",
                                          "note": "MFMA-only loop, 16x16x32 bf16 (the 32x32x16 form the attention kernels use sustains about 13 % less), N(0,1) operands, two wavefronts per SIMD"},
            "mfma_bf16_operands_that_change": {"value": round(mfma_fresh_tf, 1), "unit": "TFLOP/s",
                                               "note": "the same loop with eight A and eight B fragments per lane taken in the order of an 8 x 8 block of "
                                                       "output tiles, so that every MFMA's inputs differ from the one before as in a product of real "
                                                       "matrices: what a GEMM-shaped kernel can be held against at the chip's power limit"},
            "hbm_streaming_read": {"value": round(rd_gbps, 1), "unit": "GB/s",
                                   "note": "3 GiB read once by 2048 wavefronts, 16 KiB per wavefront in flight"}}
        log(f"[bench] attainable: MFMA-only loop {mfma_tf:.0f} TFLOP/s ({mfma_fresh_tf:.0f} with operands that change from one MFMA to the next), "
            f"streaming read {rd_gbps:.0f} GB/s")
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

    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
