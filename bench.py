#!/usr/bin/env python3
"""Benchmark of the ring-step attention path on one MI355X.

One "step" is one pass of the whole hot path for the simulated rank: cp x (step forward
fused with Update) + cast to the stored activation type + delta + cp x step backward,
every K/V chunk resident in HBM, launches back to back on one stream.

Prints ONE JSON line: fwd+bwd TFLOP/s (14*d FLOP per visible (query, key) pair per q
head: 4d forward, 10d backward including the recomputation the method needs), the MFMA
roofline of the dominant kernel (the dK/dV kernel of the backward step, timed with events
around a rotating sample of its launches inside the timed region: every event costs a few
microseconds of stream time, so bracketing all launches would slow the pass by ~4 %), and
the fp64 oracle timed on the host cores on a bounded sample of the same workload.  Extras,
measured after the timed region: every kernel bracketed, the pass replayed from a captured
graph, the step classes, Update alone, the two-buffer replay, the layout steps, the matrix
cores alone.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this script (summaries under profiles/), scaled by the same counters' reading for a copy kernel
# of known size; null for workloads that were not profiled.
TRAFFIC: dict = {"mha7b_32k": 77.7e6}  # 34.1 MiB read + 40.0 MiB written per bwd_dkv launch (average of the eight steps)


def pairs_per_head(cfg) -> int:
    L = cfg.L
    return L * (L + 1) // 2 + (cfg.cp - 1) * (L * L // 2)


def auto_cpu_rows(cfg) -> int:
    """Rows of the oracle sample for about 15 s of host work (the oracle does ~8e7 (row, key) pairs per second)."""
    return int(max(64, min(cfg.L, 1.2e9 / (cfg.hq * cfg.S))))


def cpu_baseline(cfg, inp, budget_rows: int):
    """Time the oracle as it stands (numpy fp64, its BLAS threads) on a row sample."""
    import numpy as np
    import oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    rng = np.random.default_rng(0)
    rows = np.sort(rng.choice(cfg.L, size=min(budget_rows, cfg.L), replace=False))
    pos_q = orc.zigzag_positions(cfg.cp, cfg.rank, cfg.c)[rows]
    pos_k = np.arange(cfg.S)
    t0 = time.perf_counter()
    orc.attention_backward(inp["q"][:, rows], inp["k_all"], inp["v_all"], inp["d_out"][:, rows], pos_q, pos_k, cfg.scale)
    dt = time.perf_counter() - t0
    pairs = int((pos_q + 1).sum()) * cfg.hq
    return {
        "value": 14.0 * cfg.d * pairs / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
        "sample": f"{len(rows)} of {cfg.L} local rows x {cfg.hq} heads x all {cfg.S} keys, fwd+bwd, {dt:.1f} s",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed passes (default: 200 for the 32K shape, fewer for the long ones)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed passes before them (default: as many as --steps' default: the clock needs ~0.3 s of load to settle)")
    ap.add_argument("--config", type=int, default=1, help="index into workloads.CONFIGS (1 = 7B MHA shard, 32K)")
    ap.add_argument("--cpu-rows", type=int, default=-1,
                    help="rows of the oracle sample (0: skip the CPU baseline; -1: sized for about 15 s of host work)")
    ap.add_argument("--unfused", action="store_true", help="run Attention and Update as separate kernels")
    ap.add_argument("--rank", type=int, default=None,
                    help="simulated rank of the ring (default: the workload's, rank 0); later ranks see more "
                         "steps in which both local chunks attend the visiting chunk's early half")
    ap.add_argument("--dtype", choices=["bf16", "fp16"], default=None,
                    help="storage type of q, k, v, o, d_o (default: the workload's, bf16); fp16 runs the same kernels "
                         "with the fp16 matrix instruction (same 2.5 PFLOP/s peak)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="launch only device-to-device copies of 256 MiB (reference for the HBM byte counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures the per-device ring step on ONE GPU; --gpus > 1 is not part of this build "
                 "(the ring is replayed on one device, there are no collectives)")

    import torch
    import paper_2406_18485_amd as P
    from gpu_harness import Replayed
    from workloads import CONFIGS, make_inputs

    cfg = CONFIGS[args.config]
    # default pass counts: about 0.3 s of load before the timed region (the clock climbs from idle
    # for that long; 10 warm-up passes of the 32K shape read 1 % low), about as much inside it
    passes = {0: 200, 1: 200, 2: 32, 3: 10, 4: 4}.get(args.config, 10)
    if args.steps is None:
        args.steps = passes
    if args.warmup is None:
        args.warmup = passes
    if args.rank is not None:
        if not 0 <= args.rank < cfg.cp:
            sys.exit(f"--rank must be in [0, {cfg.cp})")
        cfg = cfg.on_rank(args.rank)
    if args.dtype and cfg.dtype != "fp32":
        import dataclasses
        cfg = dataclasses.replace(cfg, dtype=args.dtype)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.copy_calibration:
        # one elementwise copy kernel reads 256 MiB and writes 256 MiB per launch
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_launch": src.numel() * 4,
                                               "bytes_written_per_launch": src.numel() * 4, "launches": 8}}))
        return
    inp = make_inputs(cfg)
    run = Replayed(cfg, inp)
    rep, s = run.rep, run.rep.shape
    fuse = not args.unfused

    desc0 = P.make_desc(batch=1, n_q_heads=s.hq, n_kv_heads=s.hkv, head_dim=s.d, q_len=s.L, kv_len=s.L,
                        dtype=s.dtype, softmax_scale=s.scale)
    step_desc = [P.make_desc(batch=1, n_q_heads=s.hq, n_kv_heads=s.hkv, head_dim=s.d, q_len=s.L, kv_len=s.L,
                             dtype=s.dtype, softmax_scale=s.scale, causal=True, chunk_len=s.c,
                             q_chunk=st["q_chunk"], kv_chunk=st["kv_chunk"]) for st in rep.plan]
    E = lambda: torch.cuda.Event(enable_timing=True)

    def backward_step(i, flags):
        src = rep.plan[i]["src_rank"]
        d = step_desc[i]
        d.flags = flags
        P.attn_step_bwd(d, run.q, run.k_by_src[src], run.v_by_src[src], None, run.d_o, rep.lse, rep.delta,
                        None if flags & P.BWD_ONLY_DKV else rep.dq,
                        None if flags & P.BWD_ONLY_DQ else rep.dk[src], None if flags & P.BWD_ONLY_DQ else rep.dv[src],
                        rep.workspace)

    def one_pass(sampled=(), every=None):
        """One pass of the path.  `sampled`: {step: (ev0, ev1)} brackets the dK/dV kernel of those
        backward micro-steps with events (the step is then issued as its two halves); `every`: an event
        dictionary that brackets the forward replay and both halves of every backward micro-step."""
        if every:
            every["fwd0"].record()
        rep.forward(run.q, run.k_by_src, run.v_by_src, fuse_merge=fuse)
        if every:
            every["fwd1"].record()
        P.bwd_delta(desc0, rep.o, run.d_o, rep.delta)
        rep.dq.zero_()
        for i in range(cfg.cp):
            if every:
                every["bwd"][i][0].record()
                backward_step(i, P.BWD_ONLY_DKV)
                every["bwd"][i][1].record()
                backward_step(i, P.BWD_ONLY_DQ)
                every["bwd"][i][2].record()
            elif i in sampled:
                sampled[i][0].record()
                backward_step(i, P.BWD_ONLY_DKV)
                sampled[i][1].record()
                backward_step(i, P.BWD_ONLY_DQ)
            else:
                backward_step(i, 0)

    # Every event costs a gap of a few microseconds on the stream, so the timed region brackets only
    # the dominant kernel, and only on a rotating sample of the micro-steps: pass p times the
    # dK/dV kernel of the steps i with i = p (mod max(steps, cp)) folded onto the steps, so that every step
    # is sampled equally often (when steps is a multiple of cp, or smaller than cp).
    def sample_of(pass_no):
        if args.steps >= cfg.cp:
            return [pass_no % cfg.cp]
        return [i for i in range(cfg.cp) if i % args.steps == pass_no % args.steps]

    for _ in range(args.warmup):
        one_pass()
    torch.cuda.synchronize()
    samples = [{i: (E(), E()) for i in sample_of(pno)} for pno in range(args.steps)]
    t0 = time.perf_counter()
    for pno in range(args.steps):
        one_pass(sampled=samples[pno])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ms_per_step = dt / args.steps * 1e3
    pairs = pairs_per_head(cfg) * cfg.hq
    tflops = 14.0 * cfg.d * pairs / (dt / args.steps) / 1e12
    # dominant kernel: the dK/dV kernel of the backward micro-step.  Its algorithmic work is four of
    # the backward's five matrix products (S, dP, dV, dK): 8*d FLOP per visible pair.  Average launch
    # duration: mean over the micro-steps of the mean of each step's samples.
    per_step = {}
    for smp in samples:
        for i, (a, b) in smp.items():
            per_step.setdefault(i, []).append(a.elapsed_time(b))
    assert len(per_step) == cfg.cp, "every micro-step must have been sampled"
    dkv_launch_ms = sum(sum(v) / len(v) for v in per_step.values()) / cfg.cp
    dkv_ms = dkv_launch_ms * cfg.cp
    dkv_tflops = 8.0 * cfg.d * pairs / (dkv_ms * 1e-3) / 1e12

    # ---- every kernel bracketed (costs ~4 % of the pass: measured outside the timed region) ----------
    def new_events():
        return {"fwd0": E(), "fwd1": E(), "bwd": [(E(), E(), E()) for _ in rep.plan]}
    n_inst = 3
    events = [new_events() for _ in range(n_inst)]
    t1 = time.perf_counter()
    for ev in events:
        one_pass(every=ev)
    torch.cuda.synchronize()
    instrumented_ms = (time.perf_counter() - t1) / n_inst * 1e3
    fwd_ms = sum(e["fwd0"].elapsed_time(e["fwd1"]) for e in events) / n_inst
    dkv_all_ms = sum(a.elapsed_time(b) for e in events for a, b, _ in e["bwd"]) / n_inst
    dq_ms = sum(b.elapsed_time(c) for e in events for _, b, c in e["bwd"]) / n_inst
    bwd_ms = dkv_all_ms + dq_ms
    per_kernel = {
        "note": f"every launch bracketed with events in {n_inst} extra passes after the timed region "
                f"({round(instrumented_ms, 4)} ms per such pass)",
        "fwd_kernel": {"flop_per_pair": "4*d", "avg_launch_ms": round(fwd_ms / cfg.cp, 4),
                       "tflops": round(4.0 * cfg.d * pairs / (fwd_ms * 1e-3) / 1e12, 1)},
        "bwd_dkv_kernel": {"flop_per_pair": "8*d", "avg_launch_ms": round(dkv_all_ms / cfg.cp, 4),
                           "tflops": round(8.0 * cfg.d * pairs / (dkv_all_ms * 1e-3) / 1e12, 1)},
        "dq_kernel": {"flop_per_pair": "6*d (S and dP recomputed)", "avg_launch_ms": round(dq_ms / cfg.cp, 4),
                      "tflops": round(6.0 * cfg.d * pairs / (dq_ms * 1e-3) / 1e12, 1)},
    }
    # the same pass replayed from a captured graph (no host launches; extra, never `value`)
    graph_ms = None
    try:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            one_pass()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                one_pass()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = round((time.perf_counter() - t2) / args.steps * 1e3, 4)
    except Exception as exc:  # a capture failure must not cost the benchmark line
        graph_ms = f"capture failed: {exc}"
    # ---- extra figures, measured after the timed region ------------------------------------
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    # per step class (rank 0: step 0 holds the own chunk = the diagonal step, the others two FULL blocks)
    def cls_ms(sel):
        idx = [i for i, st in enumerate(rep.plan) if sel(st)]
        if not idx:
            return None
        tot = sum(e["bwd"][i][0].elapsed_time(e["bwd"][i][2]) for e in events for i in idx)
        return round(tot / (len(idx) * n_inst), 4)
    step_classes = {"bwd_ms_diagonal_step": cls_ms(lambda st: st["src_rank"] == cfg.rank),
                    "bwd_ms_other_steps": cls_ms(lambda st: st["src_rank"] != cfg.rank)}
    # Update as a kernel of its own (HBM-bound): 3 x 4 x d + 3 x 4 bytes per merged row
    rows = cfg.hq * cfg.L
    blk_out, blk_lse = torch.randn(rows, cfg.d, device="cuda:0"), torch.randn(rows, device="cuda:0")
    run_out, run_lse = torch.randn(rows, cfg.d, device="cuda:0"), torch.randn(rows, device="cuda:0")
    merge_ms = timed(lambda: P.lse_merge(rows, cfg.d, run_out, run_lse, blk_out, blk_lse), 20)
    merge = {"rows": rows, "ms": round(merge_ms, 4), "bytes_per_row": 12 * cfg.d + 12,
             "GB_per_s": round(rows * (12 * cfg.d + 12) / (merge_ms * 1e-3) / 1e9, 1), "hbm_peak_GB_per_s": 8000}
    # forward with the receive buffers of Alg. 2 (device-to-device copies on two side streams stand in
    # for the inner- and outer-ring transfers) against the forward over resident chunks
    fwd_resident_ms = timed(lambda: rep.forward(run.q, run.k_by_src, run.v_by_src), 5)
    fwd_buffers_ms = timed(lambda: rep.forward_two_buffers(run.q, run.k_by_src, run.v_by_src), 5)
    stage_k = torch.empty_like(run.k_by_src[0])
    stage_v = torch.empty_like(run.v_by_src[0])
    def copies():
        for st in rep.plan:
            stage_k.copy_(run.k_by_src[st["src_rank"]], non_blocking=True)
            stage_v.copy_(run.v_by_src[st["src_rank"]], non_blocking=True)
    copies_ms = timed(copies, 5)
    two_buffers = {"fwd_ms_resident": round(fwd_resident_ms, 4), "fwd_ms_two_buffers": round(fwd_buffers_ms, 4),
                   "copies_alone_ms": round(copies_ms, 4),
                   "exposed_transfer_ms": round(max(0.0, fwd_buffers_ms - fwd_resident_ms), 4),
                   "chunk_MiB": round(run.k_by_src[0].numel() * run.k_by_src.element_size() * 2 / 2**20, 1)}
    # layout steps either side of the ring (HBM-bound, every byte read once and written once):
    # 32 heads x 4096 tokens x 128 bf16 into 4 head-group messages and back into the ring layout,
    # and the gradient reduction of 4-fold replicated KV heads
    s_tok, Hh, dd, hp = 4096, 32, 128, 4
    hl = Hh // hp
    xin = torch.zeros(s_tok, Hh, dd, dtype=torch.bfloat16, device="cuda:0")
    msg = torch.zeros(hp, hl, s_tok, dd, dtype=torch.bfloat16, device="cuda:0")
    loc = torch.zeros(hl, hp * s_tok, dd, dtype=torch.bfloat16, device="cuda:0")
    nbytes = xin.numel() * 2
    pack_ms = timed(lambda: P.permute_rows((hp, hl, s_tok), (hl * dd * 2, dd * 2, Hh * dd * 2),
                                           (hl * s_tok * dd * 2, s_tok * dd * 2, dd * 2), dd * 2, xin, msg), 20)
    unpack_ms = timed(lambda: P.permute_rows((hp, hl, s_tok), (hl * s_tok * dd * 2, s_tok * dd * 2, dd * 2),
                                             (s_tok * dd * 2, hp * s_tok * dd * 2, dd * 2), dd * 2, msg, loc), 20)
    gin = torch.zeros(8 * 4, s_tok * dd, device="cuda:0")
    gout = torch.zeros(8, s_tok * dd, device="cuda:0")
    red_ms = timed(lambda: P.reduce_replicas(8, 4, s_tok * dd, gin, gout), 20)
    layout = {"pack_heads_GB_per_s": round(2 * nbytes / (pack_ms * 1e-3) / 1e9, 1),
              "unpack_tokens_GB_per_s": round(2 * nbytes / (unpack_ms * 1e-3) / 1e9, 1),
              "reduce_replicas_GB_per_s": round((gin.numel() + gout.numel()) * 4 / (red_ms * 1e-3) / 1e9, 1),
              "tensor_MiB": nbytes >> 20}
    # the matrix cores alone, at the clocks the chip really holds
    wgs, iters_probe = 256 * 8, 4000
    sink = torch.empty(wgs * 256, device="cuda:0")
    probe_ms = timed(lambda: P.mfma_probe(wgs, iters_probe, sink), 3)
    mfma_sustained = wgs * 4 * iters_probe * 4 * 32768 / (probe_ms * 1e-3) / 1e12

    result = {
        "metric": "fwd+bwd ring-step attention TFLOP/s on 1 GPU; % of bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "fp16": "f16", "fp32": "f32"}[cfg.dtype], "data": "synthetic",
        "config": {"workload": cfg.name, "cp": cfg.cp, "inner_ring": cfg.w, "rank": cfg.rank, "q_heads": cfg.hq,
                   "kv_heads": cfg.hkv, "head_dim": cfg.d, "local_tokens": cfg.L, "total_seq": cfg.S,
                   "ring_steps": cfg.cp, "update": "fused" if fuse else "separate kernel",
                   "flop_convention": "14*d per visible pair per q head (4d fwd + 10d bwd)"},
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "tflops_12d_convention": round(tflops * 12.0 / 14.0, 2),
        "roofline": {"bound": "mfma", "kernel": "bwd_dkv_kernel (dK/dV half of one backward micro-step)",
                     "achieved": round(dkv_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(dkv_tflops / PEAK_BF16_TFLOPS, 4), "traffic": TRAFFIC.get(cfg.name),
                     "avg_launch_ms": round(dkv_launch_ms, 4), "launches_per_step": cfg.cp,
                     "timed_launches": sum(len(v) for v in per_step.values()),
                     "flop_per_launch": round(8.0 * cfg.d * pairs / cfg.cp)},
        "kernels": per_kernel,
        "graph_replay_ms_per_step": graph_ms,
        "step_classes": step_classes,
        "merge_only": merge,
        "layout_steps": layout,
        "two_buffer_replay": two_buffers,
        "mfma_only_probe_tflops": round(mfma_sustained, 1),
        "pct_of_mfma_only_probe": round(100.0 * tflops / mfma_sustained, 2),
        "fwd_ms": round(fwd_ms, 4), "bwd_ms": round(bwd_ms, 4),
    }
    cpu_rows = auto_cpu_rows(cfg) if args.cpu_rows < 0 else args.cpu_rows
    if cpu_rows > 0:
        result["cpu_baseline"] = cpu_baseline(cfg, inp, cpu_rows)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
