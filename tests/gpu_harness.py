"""Glue for the GPU parity tests: upload seeded inputs, replay the ring through the C ABI,
fetch results, and evaluate the fp64 oracle on the same bits."""
from __future__ import annotations

import numpy as np
import torch

import oracle as orc
import paper_2406_18485_amd as P
from paper_2406_18485_amd.ring import RingReplay, RingShape
from workloads import RingConfig, gather_chunks, make_inputs

TOL_O = 2e-2      # max-abs bound on O, dQ, dK, dV (bf16 inputs, fp32 accumulation)
TOL_LSE = 1e-3    # max-abs bound on LSE

DEV = "cuda:0"


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == "bf16":
        return t.to(torch.bfloat16).to(DEV)   # exact: values are bf16-representable
    if dtype == "fp16":
        return t.to(torch.float16).to(DEV)    # exact likewise
    return t.to(DEV)


def workspace_for(desc) -> torch.Tensor:
    """Caller-owned scratch for one backward step of this descriptor (never an empty allocation)."""
    return torch.empty(max(P.workspace_bytes(desc), 16), dtype=torch.uint8, device=DEV)


def shape_of(cfg: RingConfig, extra_flags: int = 0) -> RingShape:
    return RingShape(cp=cfg.cp, w=cfg.w, rank=cfg.rank, hq=cfg.hq, hkv=cfg.hkv, d=cfg.d, c=cfg.c,
                     dtype={"bf16": P.BF16, "fp16": P.FP16, "fp32": P.FP32}[cfg.dtype], scale=cfg.scale,
                     extra_flags=extra_flags)


class Replayed:
    """Device tensors of one config and the results of a forward+backward replay."""

    def __init__(self, cfg: RingConfig, inputs: dict | None = None, extra_flags: int = 0):
        self.cfg = cfg
        self.inp = inputs if inputs is not None else make_inputs(cfg)
        c, cp = cfg.c, cfg.cp
        self.q = to_dev(self.inp["q"][None], cfg.dtype)
        self.d_o = to_dev(self.inp["d_out"][None], cfg.dtype)
        ks, vs = [], []
        for s in range(cp):
            ids = (s, 2 * cp - 1 - s)
            ks.append(gather_chunks(self.inp["k_all"], ids, c)[None])
            vs.append(gather_chunks(self.inp["v_all"], ids, c)[None])
        self.k_by_src = to_dev(np.stack(ks), cfg.dtype)
        self.v_by_src = to_dev(np.stack(vs), cfg.dtype)
        self.rep = RingReplay(shape_of(cfg, extra_flags), DEV)

    def run(self, fuse_merge=True, backward=True):
        self.rep.forward(self.q, self.k_by_src, self.v_by_src, fuse_merge=fuse_merge)
        if backward:
            self.rep.backward(self.q, self.k_by_src, self.v_by_src, self.d_o)
        torch.cuda.synchronize()
        return self

    # results on the host, in the oracle's layout
    def out(self):
        return self.rep.out[0].double().cpu().numpy()

    def lse(self):
        return self.rep.lse[0].double().cpu().numpy()

    def o_stored(self):
        return self.rep.o[0].double().cpu().numpy()

    def dq(self):
        return self.rep.dq[0].double().cpu().numpy()

    def dkv_global(self):
        """dK, dV scattered back to global key order [hkv, S, d]."""
        cfg = self.cfg
        dk = np.zeros((cfg.hkv, cfg.S, cfg.d))
        dv = np.zeros_like(dk)
        for s in range(cfg.cp):
            pos = orc.zigzag_positions(cfg.cp, s, cfg.c)
            dk[:, pos] = self.rep.dk[s, 0].double().cpu().numpy()
            dv[:, pos] = self.rep.dv[s, 0].double().cpu().numpy()
        return dk, dv


def oracle_full(cfg: RingConfig, inp: dict):
    pos_q = orc.zigzag_positions(cfg.cp, cfg.rank, cfg.c)
    pos_k = np.arange(cfg.S)
    dq, dk, dv, out, lse, delta = orc.attention_backward(inp["q"], inp["k_all"], inp["v_all"], inp["d_out"],
                                                        pos_q, pos_k, cfg.scale)
    return dict(out=out, lse=lse, dq=dq, dk=dk, dv=dv, delta=delta)


def max_abs(a, b):
    return float(np.max(np.abs(np.asarray(a) - np.asarray(b)))) if np.asarray(a).size else 0.0


def check_full(run: Replayed, ref: dict, tol_o=TOL_O, tol_lse=TOL_LSE, backward=True):
    errs = {"out": max_abs(run.out(), ref["out"]), "lse": max_abs(run.lse(), ref["lse"]),
            "o_stored": max_abs(run.o_stored(), ref["out"])}
    if backward:
        dk, dv = run.dkv_global()
        errs.update(dq=max_abs(run.dq(), ref["dq"]), dk=max_abs(dk, ref["dk"]), dv=max_abs(dv, ref["dv"]))
    print(f"[parity] {run.cfg.name}: " + " ".join(f"{k}={v:.3e}" for k, v in errs.items()), flush=True)
    assert errs["lse"] <= tol_lse, errs
    for k, v in errs.items():
        if k != "lse":
            assert v <= tol_o, errs
    assert np.isfinite(run.out()).all()
    if backward:
        # the later half of an earlier rank's chunk pair lies after every local row: no gradient at all
        c = run.cfg.c
        for s in range(run.cfg.rank):
            assert float(run.rep.dk[s, :, :, c:].abs().max()) == 0.0 and float(run.rep.dv[s, :, :, c:].abs().max()) == 0.0
    return errs
