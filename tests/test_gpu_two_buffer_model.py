"""The two-buffer forward replay (Alg. 2's inner- and outer-ring receive buffers, copies on side streams) against
the time model of Sec. "P2P Communication Analysis": with the measured micro-step time as T_comp (fitted through
alpha of Sec. "Computation Analysis") and the measured copy rate as the link bandwidth, loong_cost_model gives
T_inner_ring = A (w - 1) + B per outer step, i.e. the forward time under perfect overlap.  No schedule can beat
that, and one that overlaps at all must stay below the model plus every transfer paid in full."""
import pytest
import torch

import paper_2406_18485_amd as P
from gpu_harness import Replayed
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu

MODEL_D, MODEL_H = 4096, 32   # the 7B shape behind the local head counts (head_dim 128)


def _timed(fn, reps):
    fn()
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(3):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b) / reps * 1e-3)
    return best


@pytest.mark.parametrize("idx,c", [(3, 2048), (2, 4096)])
def test_two_buffer_forward_time_lies_between_the_model_and_unoverlapped_transfers(idx, c):
    cfg = CONFIGS[idx].shrunk(c)
    run = Replayed(cfg, make_inputs(cfg))
    rep = run.rep
    sink = torch.empty(2048 * 256, device="cuda:0")
    for _ in range(40):                      # settle the clock
        P.mfma_probe(2048, 2000, sink)
    t_resident = _timed(lambda: rep.forward(run.q, run.k_by_src, run.v_by_src), 10)
    t_buffers = _timed(lambda: rep.forward_two_buffers(run.q, run.k_by_src, run.v_by_src), 10)
    stage_k, stage_v = torch.empty_like(run.k_by_src[0]), torch.empty_like(run.v_by_src[0])

    def copies():
        for st in rep.plan:
            stage_k.copy_(run.k_by_src[st["src_rank"]], non_blocking=True)
            stage_v.copy_(run.v_by_src[st["src_rank"]], non_blocking=True)
    t_copies = _timed(copies, 10)

    d_hp = MODEL_H // cfg.hq
    d_sp = d_hp * cfg.cp
    h_kv = MODEL_H if cfg.hkv == cfg.hq else 8
    chunk_bytes = 2 * run.k_by_src[0].numel() * run.k_by_src.element_size()
    alpha = (t_resident / cfg.cp) * cfg.cp * d_sp / (float(cfg.S) ** 2 * MODEL_D)
    bw = chunk_bytes / (t_copies / cfg.cp)
    m = P.cost_model(S=float(cfg.S), D=float(MODEL_D), H=MODEL_H, H_kv=h_kv, d_hp=d_hp, d_cp=cfg.cp, w=cfg.w, alpha_fwd=alpha,
                     bw_p2p_inner=bw, bw_p2p_outer=bw, bw_alltoall=bw, latency=0.0)
    assert m["size_kv"] == chunk_bytes                                   # the model's Size(kv) is the chunk that is copied
    assert abs(m["t_comp_fwd"] - t_resident / cfg.cp) < 1e-9
    predicted = m["t_inner_ring_fwd"] * (cfg.cp // cfg.w)
    print(f"[two buffers] {cfg.name}: resident {t_resident * 1e3:.3f} ms, two buffers {t_buffers * 1e3:.3f} ms, copies alone "
          f"{t_copies * 1e3:.3f} ms, model {predicted * 1e3:.3f} ms (T_comp {m['t_comp_fwd'] * 1e6:.1f} us, T_p2p "
          f"{m['t_p2p_inner_fwd'] * 1e6:.1f} us per micro-step)", flush=True)
    assert t_buffers >= 0.93 * predicted                                 # nothing beats perfect overlap (7 % timing noise)
    assert t_buffers <= predicted + t_copies + 0.10 * predicted + 1e-4   # and the transfers are at worst paid in full
