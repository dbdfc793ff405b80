#!/usr/bin/env python3
"""Benchmark of the ring-step attention path on one MI355X.

One "step" is one pass of the whole hot path for the simulated rank: cp x (step forward
fused with Update) + cast to the stored activation type + delta + cp x step backward,
every K/V chunk resident in HBM, launches back to back on one stream.

The default workload is the largest one-GPU shape (the 1M-token shard); --config picks
another.  Prints ONE JSON line: fwd+bwd TFLOP/s (14*d FLOP per visible (query, key) pair
per q head: 4d forward, 10d backward including the recomputation the method needs), the
MFMA roofline of the dominant kernel (the dK/dV kernel of the backward step, timed with
events around a rotating sample of its launches inside the timed region: every event costs
a few microseconds of stream time, so bracketing all launches would slow the pass), and the
fp64 oracle timed on the host cores on a bounded sample of the same workload.  Extras,
measured after the timed region: every kernel bracketed, the pass replayed from a captured
graph, the step classes, Update alone, the two-buffer replay against the performance model
fed with the measured step and copy times, the model's best grid for the paper's 64-GPU
setting, the layout steps, the matrix cores alone, and short runs of the other 7B shapes.
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
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the dominant kernel (average over the micro-steps of a pass) from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script (summaries under profiles/), scaled
# by the same counters' reading for a copy kernel of known size; null for workloads not profiled.
TRAFFIC: dict = {
    "mha7b_32k": 77.7e6,    # 34.1 MiB read + 40.0 MiB written
    "gqa7b_128k": 208.3e6,  # 146.6 MiB read + 52.0 MiB written (every step parks partial sums)
    "dring_256k": 339.0e6,  # 195.3 MiB read + 128.0 MiB written
    "long_1m": 557.4e6,     # 497.6 MiB read + 34.0 MiB written (each of the eight L2s streams Q and dO once;
                            # the diagonal step alone reads 7.25 GiB)
}

# model dimensions behind the local shapes (LLaMA2-7B: hidden 4096, 32 heads; 8 kv heads for GQA)
MODEL_D, MODEL_H = 4096, 32


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
    rate = 14.0 * cfg.d * pairs / dt / 1e12
    whole = 14.0 * cfg.d * pairs_per_head(cfg) * cfg.hq / 1e12 / rate
    sample = f"{len(rows)} of {cfg.L} local rows x {cfg.hq} heads x all {cfg.S} keys, fwd+bwd, {dt:.1f} s"
    if len(rows) < cfg.L:
        sample += f"; the whole workload at this rate: {whole:.0f} s (extrapolated)"
    return {"value": rate, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle", "sample": sample}


class Bench:
    """Device tensors, descriptors and the launch sequence of one workload."""

    def __init__(self, cfg, fuse=True):
        import torch
        import paper_2406_18485_amd as P
        from gpu_harness import Replayed
        from workloads import make_inputs
        self.torch, self.P, self.cfg, self.fuse = torch, P, cfg, fuse
        self.inp = make_inputs(cfg)
        self.run = Replayed(cfg, self.inp)
        self.rep, s = self.run.rep, self.run.rep.shape
        self.desc0 = P.make_desc(batch=1, n_q_heads=s.hq, n_kv_heads=s.hkv, head_dim=s.d, q_len=s.L, kv_len=s.L,
                                 dtype=s.dtype, softmax_scale=s.scale)
        self.step_desc = [P.make_desc(batch=1, n_q_heads=s.hq, n_kv_heads=s.hkv, head_dim=s.d, q_len=s.L, kv_len=s.L,
                                      dtype=s.dtype, softmax_scale=s.scale, causal=True, chunk_len=s.c,
                                      q_chunk=st["q_chunk"], kv_chunk=st["kv_chunk"]) for st in self.rep.plan]
        self.pairs = pairs_per_head(cfg) * cfg.hq

    def event(self):
        return self.torch.cuda.Event(enable_timing=True)

    def backward_step(self, i, flags):
        P, run, rep = self.P, self.run, self.rep
        src = rep.plan[i]["src_rank"]
        d = self.step_desc[i]
        d.flags = flags
        P.attn_step_bwd(d, run.q, run.k_by_src[src], run.v_by_src[src], None, run.d_o, rep.lse, rep.delta,
                        None if flags & P.BWD_ONLY_DKV else rep.dq,
                        None if flags & P.BWD_ONLY_DQ else rep.dk[src], None if flags & P.BWD_ONLY_DQ else rep.dv[src],
                        rep.workspace)

    def one_pass(self, sampled=(), every=None):
        """One pass of the path.  `sampled`: {step: (ev0, ev1)} brackets the dK/dV kernel of those
        backward micro-steps with events (the step is then issued as its two halves); `every`: an event
        dictionary that brackets the forward replay and both halves of every backward micro-step."""
        P, run, rep = self.P, self.run, self.rep
        if every:
            every["fwd0"].record()
        rep.forward(run.q, run.k_by_src, run.v_by_src, fuse_merge=self.fuse)
        if every:
            every["fwd1"].record()
        P.bwd_delta(self.desc0, rep.o, run.d_o, rep.delta)
        rep.dq.zero_()
        for i in range(self.cfg.cp):
            if every:
                every["bwd"][i][0].record()
                self.backward_step(i, P.BWD_ONLY_DKV)
                every["bwd"][i][1].record()
                self.backward_step(i, P.BWD_ONLY_DQ)
                every["bwd"][i][2].record()
            elif i in sampled:
                sampled[i][0].record()
                self.backward_step(i, P.BWD_ONLY_DKV)
                sampled[i][1].record()
                self.backward_step(i, P.BWD_ONLY_DQ)
            else:
                self.backward_step(i, 0)

    def timed_passes(self, steps, warmup):
        """`warmup` untimed passes, then `steps` timed ones with the dominant kernel bracketed on a rotating
        sample of the micro-steps: pass p times the dK/dV kernel of the steps i with i = p (mod max(steps, cp))
        folded onto the steps, so that every step is sampled equally often (when steps is a multiple of cp, or
        smaller than cp).  Returns (seconds per pass, average dK/dV launch in ms, timed launches)."""
        torch, cp = self.torch, self.cfg.cp

        def sample_of(pass_no):
            if steps >= cp:
                return [pass_no % cp]
            return [i for i in range(cp) if i % steps == pass_no % steps]

        for _ in range(warmup):
            self.one_pass()
        torch.cuda.synchronize()
        samples = [{i: (self.event(), self.event()) for i in sample_of(pno)} for pno in range(steps)]
        t0 = time.perf_counter()
        for pno in range(steps):
            self.one_pass(sampled=samples[pno])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        per_step = {}
        for smp in samples:
            for i, (a, b) in smp.items():
                per_step.setdefault(i, []).append(a.elapsed_time(b))
        # mean over the micro-steps of the mean of each step's samples (steps never sampled, possible only
        # when --steps is smaller than cp would need, are left out of the mean)
        dkv_launch_ms = sum(sum(v) / len(v) for v in per_step.values()) / len(per_step)
        return dt / steps, dkv_launch_ms, sum(len(v) for v in per_step.values()), len(per_step)

    def roofline(self, dkv_launch_ms, timed_launches, steps_seen):
        cfg = self.cfg
        flop_per_launch = 8.0 * cfg.d * self.pairs / cfg.cp
        achieved = flop_per_launch / (dkv_launch_ms * 1e-3) / 1e12
        return {"bound": "mfma", "kernel": "bwd_dkv_kernel (dK/dV half of one backward micro-step)",
                "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": TRAFFIC.get(cfg.name),
                "avg_launch_ms": round(dkv_launch_ms, 4), "launches_per_step": cfg.cp,
                "timed_launches": timed_launches, "micro_steps_sampled": steps_seen,
                "flop_per_launch": round(flop_per_launch)}


def settle_clock(P, torch, seconds=0.35):
    """The shader clock climbs from idle for about 0.3 s under load: run the matrix-core probe for that long
    before anything is timed, so that a short warm-up does not read a few per cent low."""
    sink = torch.empty(2048 * 256, device="cuda:0")
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        P.mfma_probe(2048, 2000, sink)
        torch.cuda.synchronize()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed passes (default: 8 for the 1M-token shape, more for the shorter ones)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed passes before them (default: 2..20 by workload; the clock is "
                                                              "settled by a 0.35 s matrix-core load before them in any case)")
    ap.add_argument("--config", type=int, default=4, help="index into workloads.CONFIGS (4 = the 1M-token shard, the largest one-GPU shape)")
    ap.add_argument("--cpu-rows", type=int, default=-1,
                    help="rows of the oracle sample (0: skip the CPU baseline; -1: sized for about 15 s of host work)")
    ap.add_argument("--unfused", action="store_true", help="run Attention and Update as separate kernels")
    ap.add_argument("--rank", type=int, default=None,
                    help="simulated rank of the ring (default: the workload's, rank 0); later ranks see more "
                         "steps in which both local chunks attend the visiting chunk's early half")
    ap.add_argument("--dtype", choices=["bf16", "fp16"], default=None,
                    help="storage type of q, k, v, o, d_o (default: the workload's, bf16); fp16 runs the same kernels "
                         "with the fp16 matrix instruction (same 2.5 PFLOP/s peak)")
    ap.add_argument("--no-extras", action="store_true", help="skip everything after the timed region except the CPU baseline")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the short runs of the other 7B shapes")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="launch only device-to-device copies of 256 MiB (reference for the HBM byte counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures the per-device ring step on ONE GPU; --gpus > 1 is not part of this build "
                 "(the ring is replayed on one device, there are no collectives)")

    import torch
    import paper_2406_18485_amd as P
    from workloads import CONFIGS

    cfg = CONFIGS[args.config]
    default_passes = {0: (200, 20), 1: (200, 20), 2: (32, 8), 3: (10, 3), 4: (8, 2)}.get(args.config, (10, 3))
    if args.steps is None:
        args.steps = default_passes[0]
    if args.warmup is None:
        args.warmup = default_passes[1]
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

    bench = Bench(cfg, fuse=not args.unfused)
    run, rep = bench.run, bench.rep
    pairs = bench.pairs
    E = bench.event

    settle_clock(P, torch)
    sec_per_pass, dkv_launch_ms, timed_launches, steps_seen = bench.timed_passes(args.steps, args.warmup)
    ms_per_step = sec_per_pass * 1e3
    tflops = 14.0 * cfg.d * pairs / sec_per_pass / 1e12

    result = {
        "metric": "fwd+bwd ring-step attention TFLOP/s on 1 GPU; % of bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "fp16": "f16", "fp32": "f32"}[cfg.dtype], "data": "synthetic",
        "config": {"workload": cfg.name, "cp": cfg.cp, "inner_ring": cfg.w, "rank": cfg.rank, "q_heads": cfg.hq,
                   "kv_heads": cfg.hkv, "head_dim": cfg.d, "local_tokens": cfg.L, "total_seq": cfg.S,
                   "ring_steps": cfg.cp, "update": "fused" if bench.fuse else "separate kernel",
                   "flop_convention": "14*d per visible pair per q head (4d fwd + 10d bwd)"},
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "tflops_12d_convention": round(tflops * 12.0 / 14.0, 2),
        "roofline": bench.roofline(dkv_launch_ms, timed_launches, steps_seen),
    }

    if not args.no_extras:
        # ---- every kernel bracketed (costs a few % of the pass: measured outside the timed region) ------
        def new_events():
            return {"fwd0": E(), "fwd1": E(), "bwd": [(E(), E(), E()) for _ in rep.plan]}
        n_inst = 3
        events = [new_events() for _ in range(n_inst)]
        t1 = time.perf_counter()
        for ev in events:
            bench.one_pass(every=ev)
        torch.cuda.synchronize()
        instrumented_ms = (time.perf_counter() - t1) / n_inst * 1e3
        fwd_ms = sum(e["fwd0"].elapsed_time(e["fwd1"]) for e in events) / n_inst
        dkv_all_ms = sum(a.elapsed_time(b) for e in events for a, b, _ in e["bwd"]) / n_inst
        dq_ms = sum(b.elapsed_time(c) for e in events for _, b, c in e["bwd"]) / n_inst
        bwd_ms = dkv_all_ms + dq_ms
        tf = lambda flop_per_pair_over_d, ms: round(flop_per_pair_over_d * cfg.d * pairs / (ms * 1e-3) / 1e12, 1)
        result["kernels"] = {
            "note": f"every launch bracketed with events in {n_inst} extra passes after the timed region "
                    f"({round(instrumented_ms, 4)} ms per such pass); 'algorithmic' counts each of the method's "
                    "seven matrix products once (4d forward, 10d backward), 'executed' what the kernel really issues",
            "fwd_kernel": {"algorithmic_flop_per_pair": "4*d", "avg_launch_ms": round(fwd_ms / cfg.cp, 4),
                           "tflops": tf(4.0, fwd_ms)},
            "bwd_dkv_kernel": {"algorithmic_flop_per_pair": "8*d (S, dP, dV, dK)", "avg_launch_ms": round(dkv_all_ms / cfg.cp, 4),
                               "tflops": tf(8.0, dkv_all_ms)},
            "dq_kernel": {"algorithmic_flop_per_pair": "2*d (dQ; S and dP are already counted in the dK/dV kernel)",
                          "executed_flop_per_pair": "6*d (S and dP recomputed)", "avg_launch_ms": round(dq_ms / cfg.cp, 4),
                          "tflops_algorithmic": tf(2.0, dq_ms), "tflops_executed": tf(6.0, dq_ms)},
            "backward_both_kernels": {"algorithmic_flop_per_pair": "10*d", "executed_flop_per_pair": "14*d",
                                      "tflops_algorithmic": tf(10.0, bwd_ms), "tflops_executed": tf(14.0, bwd_ms)},
        }
        result["fwd_ms"], result["bwd_ms"] = round(fwd_ms, 4), round(bwd_ms, 4)
        # the same pass replayed from a captured graph (no host launches; extra, never `value`)
        try:
            side = torch.cuda.Stream()
            with torch.cuda.stream(side):
                bench.one_pass()
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    bench.one_pass()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for _ in range(args.steps):
                g.replay()
            torch.cuda.synchronize()
            result["graph_replay_ms_per_step"] = round((time.perf_counter() - t2) / args.steps * 1e3, 4)
        except Exception as exc:  # a capture failure must not cost the benchmark line
            result["graph_replay_ms_per_step"] = f"capture failed: {exc}"

        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            a, b = E(), E()
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
        result["step_classes"] = {"bwd_ms_diagonal_step": cls_ms(lambda st: st["src_rank"] == cfg.rank),
                                  "bwd_ms_earlier_sources": cls_ms(lambda st: st["src_rank"] < cfg.rank),
                                  "bwd_ms_later_sources": cls_ms(lambda st: st["src_rank"] > cfg.rank)}
        # Update as a kernel of its own (HBM-bound): 3 x 4 x d + 3 x 4 bytes per merged row
        rows = cfg.hq * cfg.L
        blk_out, blk_lse = torch.randn(rows, cfg.d, device="cuda:0"), torch.randn(rows, device="cuda:0")
        run_out, run_lse = torch.randn(rows, cfg.d, device="cuda:0"), torch.randn(rows, device="cuda:0")
        merge_ms = timed(lambda: P.lse_merge(rows, cfg.d, run_out, run_lse, blk_out, blk_lse), 20)
        merge_gbs = rows * (12 * cfg.d + 12) / (merge_ms * 1e-3) / 1e9
        result["merge_only"] = {"rows": rows, "ms": round(merge_ms, 4), "bytes_per_row": 12 * cfg.d + 12,
                                "GB_per_s": round(merge_gbs, 1), "hbm_peak_GB_per_s": HBM_PEAK_GBS,
                                "frac_of_hbm_peak": round(merge_gbs / HBM_PEAK_GBS, 3)}
        del blk_out, blk_lse, run_out, run_lse
        # ---- forward with the receive buffers of Alg. 2 (device-to-device copies on two side streams stand in
        # for the inner- and outer-ring transfers) against the forward over resident chunks, and against the
        # performance model of Sec. "Performance Analysis" fed with what was just measured: alpha from the
        # forward micro-step, the transfer bandwidth from the copies alone.
        fwd_resident_ms = timed(lambda: rep.forward(run.q, run.k_by_src, run.v_by_src), 3)
        fwd_buffers_ms = timed(lambda: rep.forward_two_buffers(run.q, run.k_by_src, run.v_by_src), 3)
        stage_k = torch.empty_like(run.k_by_src[0])
        stage_v = torch.empty_like(run.v_by_src[0])

        def copies():
            for st in rep.plan:
                stage_k.copy_(run.k_by_src[st["src_rank"]], non_blocking=True)
                stage_v.copy_(run.v_by_src[st["src_rank"]], non_blocking=True)
        copies_ms = timed(copies, 3)
        chunk_bytes = run.k_by_src[0].numel() * run.k_by_src.element_size() * 2
        d_hp = MODEL_H // cfg.hq
        d_sp = d_hp * cfg.cp
        h_kv = MODEL_H if cfg.hkv == cfg.hq else 8
        t_step = fwd_resident_ms * 1e-3 / cfg.cp
        alpha = t_step * cfg.cp * d_sp / (float(cfg.S) ** 2 * MODEL_D)
        bw_copy = chunk_bytes / (copies_ms * 1e-3 / cfg.cp)
        model = P.cost_model(S=float(cfg.S), D=float(MODEL_D), H=MODEL_H, H_kv=h_kv, d_hp=d_hp, d_cp=cfg.cp, w=cfg.w,
                             alpha_fwd=alpha, bw_p2p_inner=bw_copy, bw_p2p_outer=bw_copy, bw_alltoall=bw_copy, latency=0.0)
        predicted_ms = model["t_inner_ring_fwd"] * (cfg.cp // cfg.w) * 1e3
        result["two_buffer_replay"] = {
            "fwd_ms_resident": round(fwd_resident_ms, 4), "fwd_ms_two_buffers": round(fwd_buffers_ms, 4),
            "copies_alone_ms": round(copies_ms, 4), "chunk_MiB": round(chunk_bytes / 2**20, 1),
            "exposed_transfer_ms_measured": round(max(0.0, fwd_buffers_ms - fwd_resident_ms), 4),
            "model": {"formula": "forward = (d_cp / w) * (A (w - 1) + B), A = max(T_comp, T_p2p_inner), B = max(T_comp, T_p2p_outer)",
                      "alpha_fwd_measured": alpha, "t_comp_fwd_ms": round(model["t_comp_fwd"] * 1e3, 4),
                      "t_p2p_ms": round(model["t_p2p_inner_fwd"] * 1e3, 4), "size_kv_MiB": round(model["size_kv"] / 2**20, 2),
                      "copy_GB_per_s": round(bw_copy / 1e9, 1), "fwd_ms_predicted": round(predicted_ms, 4),
                      "exposed_transfer_ms_predicted": round(max(0.0, predicted_ms - fwd_resident_ms), 4)},
        }
        del stage_k, stage_v
        # the model's best grid for the paper's setting (64 GPUs, 1M tokens, Sec. "Experiment Setup") on MI355X nodes,
        # with this run's alpha and ASSUMED link rates: ring hop inside a node = one xGMI link, 76.8 GB/s per
        # direction; between nodes one 400 Gb/s NIC per GPU = 50 GB/s; all-to-all inside a node = seven links
        links = dict(bw_p2p_inner=76.8e9, bw_p2p_outer=50e9, bw_alltoall=7 * 76.8e9, latency=5e-6)
        best = {}
        for name, hkv in (("mha", 32), ("gqa", 8)):
            b = P.cost_search(64, 8, S=float(1 << 20), D=float(MODEL_D), H=MODEL_H, H_kv=hkv, alpha_fwd=alpha, **links)
            best[name] = {"d_hp": b["d_hp"], "d_cp": b["d_cp"], "w": b["w"], "objective_ms": round(b["objective"] * 1e3, 2),
                          "t_seq_alltoall_ms": round(b["t_seq_alltoall"] * 1e3, 3)}
        result["cost_model_best_grid_64gpu_1m"] = {"assumed_links": links, "alpha_fwd": alpha, **best}
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
        result["layout_steps"] = {"pack_heads_GB_per_s": round(2 * nbytes / (pack_ms * 1e-3) / 1e9, 1),
                                  "unpack_tokens_GB_per_s": round(2 * nbytes / (unpack_ms * 1e-3) / 1e9, 1),
                                  "reduce_replicas_GB_per_s": round((gin.numel() + gout.numel()) * 4 / (red_ms * 1e-3) / 1e9, 1),
                                  "tensor_MiB": nbytes >> 20}
        # the matrix cores alone, at the clocks the chip really holds
        wgs, iters_probe = 256 * 8, 4000
        sink = torch.empty(wgs * 256, device="cuda:0")
        probe_ms = timed(lambda: P.mfma_probe(wgs, iters_probe, sink), 3)
        mfma_sustained = wgs * 4 * iters_probe * 4 * 32768 / (probe_ms * 1e-3) / 1e12
        result["mfma_only_probe_tflops"] = round(mfma_sustained, 1)
        result["pct_of_mfma_only_probe"] = round(100.0 * tflops / mfma_sustained, 2)
        # the same with operands drawn like the workload's q/k/v (normal * 0.5, bf16): more bits toggle,
        # the chip holds a lower clock, and that lower rate is what any kernel fed such data can reach
        gen = torch.Generator(device="cuda:0").manual_seed(7)
        operands = (torch.randn(1024, device="cuda:0", generator=gen) * 0.5).bfloat16()
        settle_clock(P, torch, 0.2)
        probe_ms = timed(lambda: P.mfma_probe(wgs, iters_probe, sink, operands), 3)
        mfma_random = wgs * 4 * iters_probe * 4 * 32768 / (probe_ms * 1e-3) / 1e12
        result["mfma_only_probe_workload_values_tflops"] = round(mfma_random, 1)
        result["pct_of_mfma_only_probe_workload_values"] = round(100.0 * tflops / mfma_random, 2)

    cpu_rows = auto_cpu_rows(cfg) if args.cpu_rows < 0 else args.cpu_rows
    if cpu_rows > 0:
        result["cpu_baseline"] = cpu_baseline(cfg, bench.inp, cpu_rows)

    # ---- the other 7B shapes, briefly (about 0.3 s of timed passes each, same launch sequence, rank 0) ----
    if not args.no_extras and not args.no_other_configs and args.rank is None and args.dtype is None and not args.unfused:
        del bench, run, rep
        torch.cuda.empty_cache()
        others = {}
        for idx, (steps, warmup) in ((1, (200, 20)), (2, (32, 4)), (3, (10, 2)), (4, (4, 1))):
            if idx == args.config:
                continue
            ob = Bench(CONFIGS[idx])
            settle_clock(P, torch, 0.2)
            sec, launch_ms, n_timed, seen = ob.timed_passes(steps, warmup)
            rate = 14.0 * ob.cfg.d * ob.pairs / sec / 1e12
            roof = ob.roofline(launch_ms, n_timed, seen)
            others[ob.cfg.name] = {"value": round(rate, 2), "pct_of_bf16_mfma_peak": round(100.0 * rate / PEAK_BF16_TFLOPS, 2),
                                   "ms_per_step": round(sec * 1e3, 4), "steps": steps, "warmup": warmup,
                                   "roofline_frac": roof["frac"], "dkv_avg_launch_ms": roof["avg_launch_ms"]}
            del ob
            torch.cuda.empty_cache()
        result["per_config"] = others
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
