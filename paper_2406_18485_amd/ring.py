"""Single-GPU replay of one device's share of Double-Ring-Attention.

The ring is simulated by visiting the K/V chunks, all resident in HBM, in the order in
which the inner and outer rings of Alg. 2 would deliver them to the simulated rank; each
visit is one call of the library's step kernels.  torch is used for device memory and
the stream only.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as B


@dataclass
class RingShape:
    cp: int
    w: int
    rank: int
    hq: int
    hkv: int
    d: int
    c: int
    dtype: int          # B.BF16 | B.FP32 | B.FP16
    scale: float
    batch: int = 1
    extra_flags: int = 0   # OR-ed into every step descriptor (e.g. binding.key_splits(n))

    @property
    def L(self) -> int:
        return 2 * self.c


def visit_plan(shape: RingShape) -> list[dict]:
    """Per micro-step: source rank, chunk ids and block classes, from the library."""
    return [B.zigzag_mask(shape.cp, shape.w, shape.rank, t) for t in range(shape.cp)]


def _desc(shape: RingShape, step: dict, flags: int) -> B.StepDesc:
    return B.make_desc(batch=shape.batch, n_q_heads=shape.hq, n_kv_heads=shape.hkv, head_dim=shape.d,
                       q_len=shape.L, kv_len=shape.L, dtype=shape.dtype, softmax_scale=shape.scale,
                       causal=True, chunk_len=shape.c, q_chunk=step["q_chunk"], kv_chunk=step["kv_chunk"],
                       flags=flags | shape.extra_flags)


class RingReplay:
    """Buffers and launch sequence of the forward and backward replay for one rank.

    k_by_src / v_by_src: [cp, batch, hkv, L, d] device tensors holding, for every source
    rank, its zigzag chunk pair (low half first).  q, d_o: [batch, hq, L, d].
    """

    def __init__(self, shape: RingShape, device="cuda:0"):
        self.shape = shape
        self.dev = torch.device(device)
        self.plan = visit_plan(shape)
        s = shape
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.store_dtype = {B.BF16: torch.bfloat16, B.FP16: torch.float16, B.FP32: torch.float32}[s.dtype]
        self.rows = s.batch * s.hq * s.L
        self.out = torch.empty(s.batch, s.hq, s.L, s.d, **f32)      # running fp32 output
        self.lse = torch.empty(s.batch, s.hq, s.L, **f32)
        self.o = torch.empty(s.batch, s.hq, s.L, s.d, dtype=self.store_dtype, device=self.dev)
        self.delta = torch.empty(s.batch, s.hq, s.L, **f32)
        self.dq = torch.empty(s.batch, s.hq, s.L, s.d, **f32)
        self.dk = torch.empty(s.cp, s.batch, s.hkv, s.L, s.d, **f32)  # per source rank
        self.dv = torch.empty(s.cp, s.batch, s.hkv, s.L, s.d, **f32)
        self.block_out = None
        self.block_lse = None
        # caller-owned scratch of the backward steps: the largest any micro-step asks for
        need = max(B.workspace_bytes(_desc(s, step, 0)) for step in self.plan)
        self.workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=self.dev)

    # ---- forward: cp x (Attention [+ Update]) then the cast to the stored activation type
    def forward(self, q, k_by_src, v_by_src, fuse_merge=True, stream=None):
        s = self.shape
        if not fuse_merge:
            B.init_running(self.rows, s.d, self.out, self.lse, stream)
            if self.block_out is None:
                self.block_out = torch.empty_like(self.out)
                self.block_lse = torch.empty_like(self.lse)
        for t, step in enumerate(self.plan):
            src = step["src_rank"]
            if fuse_merge:
                # the first visit writes the running result (rows that see nothing get the neutral
                # element), the later ones merge into it: no separate initialisation
                B.attn_step_fwd(_desc(s, step, B.FUSE_MERGE if t else 0), q, k_by_src[src], v_by_src[src],
                                self.out, self.lse, stream)
            else:
                B.attn_step_fwd(_desc(s, step, 0), q, k_by_src[src], v_by_src[src], self.block_out, self.block_lse, stream)
                B.lse_merge(self.rows, s.d, self.out, self.lse, self.block_out, self.block_lse, stream)
        B.finalize_out(self.rows, s.d, self.out, self.o, s.dtype, stream)

    # ---- backward from the stored O and LSE: delta once, then cp step kernels
    def backward(self, q, k_by_src, v_by_src, d_o, stream=None):
        s = self.shape
        self.dq.zero_()
        first = True
        for step in self.plan:
            src = step["src_rank"]
            flags = B.COMPUTE_DELTA if first else 0
            first = False
            B.attn_step_bwd(_desc(s, step, flags), q, k_by_src[src], v_by_src[src], self.o, d_o, self.lse,
                            self.delta, self.dq, self.dk[src], self.dv[src], self.workspace, stream=stream)

    # ---- forward with the receive buffers of Alg. 2: the chunk of the next micro-step arrives
    # in an inner-ring buffer while the current one is used, and the first chunk of the next
    # outer step arrives in the outer-ring buffer during the whole inner ring.  On one GPU the
    # "transfers" are device-to-device copies from the resident chunks on two side streams
    # (default priority), ordered against the step kernels with events exactly as the P2P
    # receives would be.  Result: the same (out, lse, o) as forward().
    def forward_two_buffers(self, q, k_by_src, v_by_src):
        s = self.shape
        main = torch.cuda.current_stream(self.dev)
        if not hasattr(self, "_kv_bufs"):
            shp = (s.batch, s.hkv, s.L, s.d)
            self._kv_bufs = [(torch.empty(shp, dtype=self.store_dtype, device=self.dev),
                              torch.empty(shp, dtype=self.store_dtype, device=self.dev)) for _ in range(3)]
            self._comm = (torch.cuda.Stream(self.dev), torch.cuda.Stream(self.dev))   # inner ring, outer ring
        bufs, (inner, outer) = self._kv_bufs, self._comm
        filled = [torch.cuda.Event() for _ in range(3)]
        released = [torch.cuda.Event() for _ in range(3)]

        def receive(stream, b, src):
            stream.wait_event(released[b])          # the buffer's last reader has finished
            with torch.cuda.stream(stream):
                bufs[b][0].copy_(k_by_src[src], non_blocking=True)
                bufs[b][1].copy_(v_by_src[src], non_blocking=True)
                filled[b].record(stream)

        for ev in released:
            ev.record(main)
        cur, nxt, out = 0, 1, 2
        receive(inner, cur, self.plan[0]["src_rank"])   # the own chunk
        n_outer = s.cp // s.w
        for t, step in enumerate(self.plan):
            a, b = divmod(t, s.w)
            if b == 0 and a + 1 < n_outer:
                receive(outer, out, self.plan[(a + 1) * s.w]["src_rank"])
            if b + 1 < s.w:
                receive(inner, nxt, self.plan[t + 1]["src_rank"])
            main.wait_event(filled[cur])
            B.attn_step_fwd(_desc(s, step, B.FUSE_MERGE if t else 0), q, bufs[cur][0], bufs[cur][1], self.out, self.lse)
            released[cur].record(main)
            if b + 1 < s.w:
                cur, nxt = nxt, cur
            else:
                cur, out = out, cur
        B.finalize_out(self.rows, s.d, self.out, self.o, s.dtype)
