"""The backward entry point that allocates nothing (scratch in a static device array) against
loong_attn_step_bwd with a caller-owned workspace: same kernels, same order of additions, so the
results must be bit-identical; two calls in a row, the second on a smaller input, then the
first again (the array keeps the last call's contents; every call clears what it counts in)."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2406_18485_amd as P
from gpu_harness import DEV, workspace_for

pytestmark = pytest.mark.gpu


def _problem(hq, hkv, d, c, q_chunk, kv_chunk, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    L = 2 * c
    mk = lambda *s: (torch.randn(*s, generator=g) * 0.5).to(torch.bfloat16).to(DEV)
    t = dict(q=mk(1, hq, L, d), k=mk(1, hkv, L, d), v=mk(1, hkv, L, d), o=mk(1, hq, L, d), d_o=mk(1, hq, L, d))
    t["lse"] = (torch.rand(1, hq, L, generator=g) * 2.0 + 6.0).to(DEV)
    desc = P.make_desc(batch=1, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, q_len=L, kv_len=L, dtype=P.BF16,
                       softmax_scale=1.0 / np.sqrt(d), causal=True, chunk_len=c, q_chunk=q_chunk, kv_chunk=kv_chunk,
                       flags=P.COMPUTE_DELTA)
    return desc, t


def _run(desc, t, static):
    hq, L, d = t["q"].shape[1:]
    hkv = t["k"].shape[1]
    delta = torch.empty(1, hq, L, device=DEV)
    dq = torch.zeros(1, hq, L, d, device=DEV)
    dk, dv = torch.full((1, hkv, L, d), 5.0, device=DEV), torch.full((1, hkv, L, d), 5.0, device=DEV)
    if static:
        P.attn_step_bwd_static(desc, t["q"], t["k"], t["v"], t["o"], t["d_o"], t["lse"], delta, dq, dk, dv)
    else:
        P.attn_step_bwd(desc, t["q"], t["k"], t["v"], t["o"], t["d_o"], t["lse"], delta, dq, dk, dv, workspace_for(desc))
    torch.cuda.synchronize()
    return delta, dq, dk, dv


def test_static_scratch_backward_equals_the_workspace_backward_on_two_calls_in_a_row():
    # both problems share query loops between workgroups (few key tiles): the scratch is really used
    big = _problem(8, 2, 128, 768, (3, 4), (1, 6), seed=1)      # both local chunks x the early keys: 2 heads x 6 key tiles
    small = _problem(4, 1, 64, 200, (2, 5), (2, 5), seed=2)     # the diagonal step of a smaller, ragged shape
    for desc, _ in (big, small):
        assert 0 < P.workspace_bytes(desc) <= P.STATIC_SCRATCH_BYTES
    want = [_run(*pb, static=False) for pb in (big, small)]
    got = [_run(*pb, static=True) for pb in (big, small, big)]   # in a row, on the one array
    for g, w in zip(got, want + [want[0]]):
        for a, b in zip(g, w):
            assert torch.equal(a, b)
    assert all(torch.isfinite(x).all() for x in got[0])


def test_static_scratch_backward_refuses_what_does_not_fit_and_needs_no_scratch_when_loops_are_not_shared():
    lib = P.binding.lib
    # 1 kv head x 254 key tiles, diagonal step: 4 workgroups per key tile -> more than the array holds
    huge = P.make_desc(batch=1, n_q_heads=1, n_kv_heads=1, head_dim=128, q_len=32512, kv_len=32512, dtype=P.BF16,
                       softmax_scale=0.1, causal=True, chunk_len=16256, q_chunk=(0, 3), kv_chunk=(0, 3))
    assert P.workspace_bytes(huge) > P.STATIC_SCRATCH_BYTES
    fake = [0x1000] * 3 + [None] + [0x1000] * 6
    assert lib.loong_attn_step_bwd_static(C.byref(huge), *fake, None) == P.E_UNSUPPORTED and "scratch" in P.last_error()
    # a step with many key tiles shares nothing and needs no scratch: same results again
    plain = _problem(8, 8, 128, 2048, (0, 15), (3, 12), seed=3)
    assert P.workspace_bytes(plain[0]) == 0
    for a, b in zip(_run(*plain, static=True), _run(*plain, static=False)):
        assert torch.equal(a, b)
