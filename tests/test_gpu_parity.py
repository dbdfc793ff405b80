"""GPU parity tests: the HIP path, called through the C ABI, against the fp64 oracle on the
same seeded inputs.  Bounds: max-abs 2e-2 on O, dQ, dK, dV and 1e-3 on LSE (bf16 inputs,
fp32 accumulation); fp32-storage cases are held to 2e-4 / 1e-4."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2406_18485_amd as P
from paper_2406_18485_amd import ring
from gpu_harness import (DEV, TOL_LSE, TOL_O, Replayed, check_full, max_abs, oracle_full, to_dev, workspace_for)
from workloads import CONFIGS, RingConfig, make_inputs, round_to_bf16

pytestmark = pytest.mark.gpu


def _f32(*shape, seed=0, sigma=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * sigma).astype(np.float32)


# ------------------------------------------------------------------------------ row kernels
@pytest.mark.parametrize("rows,d", [(1, 4), (37, 64), (1000, 128), (4099, 128), (513, 96), (65, 256), (3, 260)])
def test_lse_merge_matches_oracle_update(rows, d):
    out, bout = _f32(rows, d, seed=1), _f32(rows, d, seed=2)
    lse, blse = _f32(rows, seed=3, sigma=4.0), _f32(rows, seed=4, sigma=4.0)
    # neutral sides in every combination
    lse[::7] = -np.inf
    blse[::5] = -np.inf
    out[::7] = 0.0
    bout[::5] = 0.0
    ref_out, ref_lse = orc.update(out, lse, bout, blse)
    t_out, t_lse = torch.from_numpy(out).to(DEV), torch.from_numpy(lse).to(DEV)
    P.lse_merge(rows, d, t_out, t_lse, torch.from_numpy(bout).to(DEV), torch.from_numpy(blse).to(DEV))
    torch.cuda.synchronize()
    got_lse = t_lse.cpu().numpy().astype(np.float64)
    assert np.array_equal(np.isneginf(got_lse), np.isneginf(ref_lse))
    fin = np.isfinite(ref_lse)
    assert max_abs(got_lse[fin], ref_lse[fin]) < 2e-6 * max(1.0, np.abs(ref_lse[fin]).max(initial=0.0))
    assert max_abs(t_out.cpu().numpy(), ref_out) < 1e-5
    # rows that received nothing are bit-identical to what they were
    keep = np.isneginf(blse)
    assert np.array_equal(t_out.cpu().numpy()[keep], out[keep])


def test_lse_merge_zero_rows_is_a_noop():
    t = torch.zeros(4, 128, device=DEV)
    l = torch.zeros(4, device=DEV)
    P.lse_merge(0, 128, t, l, t, l)
    torch.cuda.synchronize()


def test_init_running_and_finalize():
    rows, d = 777, 128
    out = torch.full((rows, d), 3.0, device=DEV)
    lse = torch.zeros(rows, device=DEV)
    P.init_running(rows, d, out, lse)
    torch.cuda.synchronize()
    assert torch.all(out == 0) and torch.all(torch.isneginf(lse))
    x = _f32(rows, d, seed=5, sigma=3.0)
    o16 = torch.empty(rows, d, dtype=torch.bfloat16, device=DEV)
    P.finalize_out(rows, d, torch.from_numpy(x).to(DEV), o16, P.BF16)
    o32 = torch.empty(rows, d, dtype=torch.float32, device=DEV)
    P.finalize_out(rows, d, torch.from_numpy(x).to(DEV), o32, P.FP32)
    torch.cuda.synchronize()
    assert np.array_equal(o16.float().cpu().numpy(), round_to_bf16(x))   # round to nearest even, bit exact
    assert np.array_equal(o32.cpu().numpy(), x)
    x[:8, 0] = [65504.0, 65520.0, 6.0e-8, 2.0 ** -25, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, -0.0, 3.0e-5]  # fp16 edges: max, overflow, subnormals, ties
    h16 = torch.empty(rows, d, dtype=torch.float16, device=DEV)
    P.finalize_out(rows, d, torch.from_numpy(x).to(DEV), h16, P.FP16)
    torch.cuda.synchronize()
    with np.errstate(over="ignore"):
        want = x.astype(np.float16)
    assert np.array_equal(h16.cpu().numpy().view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("fp16", 128), ("fp16", 64), ("fp32", 64), ("fp32", 100)])
def test_bwd_delta_matches_rowsum(dtype, d):
    b, h, n = 2, 3, 301
    o, do = _f32(b, h, n, d, seed=6), _f32(b, h, n, d, seed=7)
    if dtype == "bf16":
        o, do = round_to_bf16(o), round_to_bf16(do)
    if dtype == "fp16":
        o, do = o.astype(np.float16).astype(np.float32), do.astype(np.float16).astype(np.float32)
    desc = P.make_desc(batch=b, n_q_heads=h, n_kv_heads=h, head_dim=d, q_len=n, kv_len=n,
                       dtype={"bf16": P.BF16, "fp16": P.FP16, "fp32": P.FP32}[dtype], softmax_scale=1.0)
    delta = torch.empty(b, h, n, device=DEV)
    P.bwd_delta(desc, to_dev(o, dtype), to_dev(do, dtype), delta)
    torch.cuda.synchronize()
    assert max_abs(delta.cpu().numpy(), orc.rowsum_delta(do, o)) < 2e-4


# ------------------------------------------------------------------------------ whole replays
def test_tiny_fp32_config_full_parity_fused_and_unfused():
    cfg = CONFIGS[0]
    inp = make_inputs(cfg)
    ref = oracle_full(cfg, inp)
    run = Replayed(cfg, inp)
    check_full(run.run(fuse_merge=True), ref, tol_o=2e-4, tol_lse=1e-4)
    fused_out = run.out().copy()
    check_full(run.run(fuse_merge=False), ref, tol_o=2e-4, tol_lse=1e-4)
    assert max_abs(fused_out, run.out()) < 1e-5


def test_tiny_config_through_the_bf16_kernels():
    cfg = RingConfig("tiny_bf16", cp=4, w=4, rank=0, hq=2, hkv=2, d=64, c=128, dtype="bf16", sigma=1.0, seed=1000)
    inp = make_inputs(cfg)
    check_full(Replayed(cfg, inp).run(), oracle_full(cfg, inp))


SMALL = [
    # hq hkv d   c   cp w rank
    (2, 2, 128, 64, 2, 2, 0),
    (2, 2, 128, 64, 2, 2, 1),
    (4, 1, 128, 200, 4, 2, 2),    # ragged chunk, GQA 4:1, double ring
    (8, 1, 64, 96, 2, 1, 1),      # GQA 8:1, head_dim 64
    (6, 2, 128, 33, 3, 3, 1),     # group of 3: no head stacking
    (2, 1, 128, 1, 2, 2, 0),      # one token per chunk
    (4, 2, 64, 257, 2, 2, 0),
    (1, 1, 128, 520, 2, 2, 1),    # several key tiles and a ragged tail
]


@pytest.mark.parametrize("hq,hkv,d,c,cp,w,rank", SMALL)
def test_bf16_small_shapes_full_parity(hq, hkv, d, c, cp, w, rank):
    cfg = RingConfig(f"small_h{hq}_{hkv}_d{d}_c{c}_cp{cp}_r{rank}", cp=cp, w=w, rank=rank, hq=hq, hkv=hkv, d=d, c=c,
                     dtype="bf16", sigma=0.7, seed=77 + c)
    inp = make_inputs(cfg)
    ref = oracle_full(cfg, inp)
    run = Replayed(cfg, inp)
    check_full(run.run(fuse_merge=True), ref)
    check_full(run.run(fuse_merge=False), ref)


def _drawn_shapes(n, seed):
    """Seeded draw of ring shapes: group sizes 1..8, both head dims, chunk lengths around the
    32-, 64- and 128-token tile edges, every ring factorisation of cp, any rank."""
    rng = np.random.default_rng(seed)
    edges = [31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 255, 256, 300]
    out = []
    for _ in range(n):
        hkv = int(rng.integers(1, 3))
        group = int(rng.choice([1, 2, 3, 4, 8]))
        cp = int(rng.choice([2, 3, 4, 6]))
        w = int(rng.choice([x for x in range(1, cp + 1) if cp % x == 0]))
        out.append((hkv * group, hkv, int(rng.choice([64, 128])), int(rng.choice(edges)), cp, w,
                    int(rng.integers(0, cp))))
    return out


@pytest.mark.parametrize("hq,hkv,d,c,cp,w,rank", _drawn_shapes(14, seed=20240626))
def test_bf16_drawn_shapes_full_parity(hq, hkv, d, c, cp, w, rank):
    cfg = RingConfig(f"drawn_h{hq}_{hkv}_d{d}_c{c}_cp{cp}w{w}_r{rank}", cp=cp, w=w, rank=rank, hq=hq, hkv=hkv,
                     d=d, c=c, dtype="bf16", sigma=0.8, seed=5 * c + rank)
    inp = make_inputs(cfg)
    check_full(Replayed(cfg, inp).run(), oracle_full(cfg, inp))


# ---- IEEE half storage: the same kernels with the fp16 matrix instruction.  Ten mantissa bits
# instead of seven: the bounds are those of bf16 cut by four (observed errors are ~8x smaller).
@pytest.mark.parametrize("hq,hkv,d,c,cp,w,rank", SMALL[2:] + _drawn_shapes(6, seed=16))
def test_fp16_shapes_full_parity(hq, hkv, d, c, cp, w, rank):
    cfg = RingConfig(f"half_h{hq}_{hkv}_d{d}_c{c}_cp{cp}w{w}_r{rank}", cp=cp, w=w, rank=rank, hq=hq, hkv=hkv, d=d, c=c,
                     dtype="fp16", sigma=0.7, seed=300 + c)
    inp = make_inputs(cfg)
    ref = oracle_full(cfg, inp)
    run = Replayed(cfg, inp)
    check_full(run.run(fuse_merge=True), ref, tol_o=TOL_O / 4, tol_lse=TOL_LSE / 4)
    check_full(run.run(fuse_merge=False), ref, tol_o=TOL_O / 4, tol_lse=TOL_LSE / 4)


@pytest.mark.parametrize("idx", [1, 2, 3])
def test_fp16_shrunken_benchmark_configs_full_parity(idx):
    import dataclasses
    cfg = dataclasses.replace(CONFIGS[idx].shrunk(320 if CONFIGS[idx].cp < 16 else 192), dtype="fp16")
    inp = make_inputs(cfg)
    check_full(Replayed(cfg, inp).run(), oracle_full(cfg, inp), tol_o=TOL_O / 4, tol_lse=TOL_LSE / 4)


def test_fp16_large_scores_stay_finite():
    """Scores far beyond the fp16 range of exp(): probabilities are formed relative to the running
    maximum in fp32 and only then rounded to half, so nothing overflows."""
    cfg = RingConfig("half_large_scores", cp=2, w=2, rank=1, hq=2, hkv=2, d=64, c=96, dtype="fp16", sigma=6.0, seed=41)
    inp = make_inputs(cfg)
    ref = oracle_full(cfg, inp)
    run = Replayed(cfg, inp).run(backward=False)
    assert np.isfinite(run.out()).all() and np.isfinite(run.lse()).all()
    check_full(run, ref, tol_o=5e-2, tol_lse=1e-2, backward=False)


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
@pytest.mark.parametrize("which_rank", ["first", "middle"])
def test_shrunken_benchmark_configs_full_parity(idx, which_rank):
    cfg = CONFIGS[idx].shrunk(320)
    if which_rank == "middle":
        cfg = cfg.on_rank(cfg.cp // 2)
    if cfg.cp >= 16:
        cfg = cfg.shrunk(192)
    inp = make_inputs(cfg)
    check_full(Replayed(cfg, inp).run(), oracle_full(cfg, inp))


def test_forward_is_bit_reproducible_and_order_of_visits_does_not_matter():
    cfg = CONFIGS[3].shrunk(256)                     # cp=16, inner ring 4
    inp = make_inputs(cfg)
    a = Replayed(cfg, inp).run(backward=True)
    out1, lse1 = a.out().copy(), a.lse().copy()
    a.run(backward=False)
    assert np.array_equal(out1, a.out()) and np.array_equal(lse1, a.lse())
    lin = Replayed(RingConfig(**{**cfg.__dict__, "w": cfg.cp}), inp).run()
    assert [s["src_rank"] for s in lin.rep.plan] != [s["src_rank"] for s in a.rep.plan]
    # P is rounded to bf16 relative to the running maximum, which depends on the visit order:
    # O agrees to bf16-rounding level, LSE (fp32 sums) to fp32-rounding level
    assert max_abs(lin.out(), out1) < 1e-3 and max_abs(lin.lse(), lse1) < 1e-4
    dk_a, dv_a = a.dkv_global()
    dk_l, dv_l = lin.dkv_global()
    assert max_abs(dk_a, dk_l) < 2e-3 and max_abs(dv_a, dv_l) < 2e-3 and max_abs(a.dq(), lin.dq()) < 2e-3


@pytest.mark.parametrize("idx,c", [(1, 320), (2, 320), (3, 192), (1, 2048), (2, 8192)])
def test_backward_is_bit_reproducible(idx, c):
    """dQ rows are owned by one thread group; dK/dV of a key tile whose query loop several workgroups share
    are summed by the last of them in a fixed order (the small shapes here all share loops; the full 32K
    shape does on its diagonal step, the full GQA shape on every step): no result depends on the order in
    which workgroups finish."""
    cfg = CONFIGS[idx].shrunk(c) if c != CONFIGS[idx].c else CONFIGS[idx]
    run = Replayed(cfg, make_inputs(cfg)).run()
    first = [t.clone() for t in (run.rep.dq, run.rep.dk, run.rep.dv)]
    for _ in range(4):
        run.rep.dk.fill_(3.0)
        run.run()
        for got, want in zip((run.rep.dq, run.rep.dk, run.rep.dv), first):
            assert torch.equal(got, want)


def test_partial_sums_of_one_launch_never_reach_the_next():
    """Workgroups that share a query loop exchange partial dK/dV through one buffer that every launch reuses.
    Two problems of the same shape and different data, run alternately, must each reproduce their own first
    results bit for bit (and those match the oracle): a partial sum left over from the other problem, read
    in place of a fresh one, would show."""
    base = CONFIGS[1].shrunk(448)
    runs = []
    for seed in (11, 12):
        cfg = RingConfig(**{**base.__dict__, "seed": seed, "name": f"{base.name}/seed{seed}"})
        inp = make_inputs(cfg)
        runs.append((Replayed(cfg, inp), oracle_full(cfg, inp)))
    firsts = []
    for run, ref in runs:
        check_full(run.run(), ref)
        firsts.append([t.clone() for t in (run.rep.dq, run.rep.dk, run.rep.dv)])
    for _ in range(3):
        for (run, _), first in zip(runs, firsts):
            run.run()
            for got, want in zip((run.rep.dq, run.rep.dk, run.rep.dv), first):
                assert torch.equal(got, want)


@pytest.mark.parametrize("idx,c", [(3, 192), (1, 128), (2, 160)])
def test_two_buffer_forward_equals_the_resident_replay(idx, c):
    """The receive-buffer schedule of Alg. 2 (inner and outer ring buffers, copies on side streams) must match the
    oracle, and be bit-identical to the replay over resident chunks: same kernels, same data, only the event
    ordering differs."""
    cfg = CONFIGS[idx].shrunk(c)
    inp = make_inputs(cfg)
    run = Replayed(cfg, inp)
    run.rep.out.fill_(7.0)
    run.rep.forward_two_buffers(run.q, run.k_by_src, run.v_by_src)
    torch.cuda.synchronize()
    check_full(run, oracle_full(cfg, inp), backward=False)
    run.rep.forward(run.q, run.k_by_src, run.v_by_src)
    torch.cuda.synchronize()
    ref = (run.rep.out.clone(), run.rep.lse.clone(), run.rep.o.clone())
    for _ in range(2):   # twice: the buffers and streams are reused
        run.rep.out.fill_(7.0)
        run.rep.forward_two_buffers(run.q, run.k_by_src, run.v_by_src)
        torch.cuda.synchronize()
        assert torch.equal(run.rep.out, ref[0]) and torch.equal(run.rep.lse, ref[1]) and torch.equal(run.rep.o, ref[2])


@pytest.mark.parametrize("idx,c", [(1, 256), (3, 192)])
def test_captured_graph_of_the_whole_pass_replays_bit_exactly(idx, c):
    """The launch sequence of a forward + backward pass (no allocation, no host synchronisation, no
    memset node: clears are fill kernels) can be captured in a HIP graph.  Every replay, with eager work of
    the program's own and synchronisations in between, must reproduce the eager results bit for bit, dK/dV
    included: both shapes share query loops between workgroups (partial sums through the caller's workspace,
    counters cleared by a kernel that is part of the captured sequence), and those are added in a fixed order."""
    cfg = CONFIGS[idx].shrunk(c)
    run = Replayed(cfg, make_inputs(cfg))
    rep = run.rep
    assert max(P.workspace_bytes(ring._desc(rep.shape, st, 0)) for st in rep.plan) > 0   # query loops are shared

    def one_pass():
        rep.forward(run.q, run.k_by_src, run.v_by_src)
        rep.backward(run.q, run.k_by_src, run.v_by_src, run.d_o)

    one_pass()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (rep.out, rep.lse, rep.o, rep.dq)]
    ref_dk, ref_dv = rep.dk.clone(), rep.dv.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        one_pass()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            one_pass()
    torch.cuda.synchronize()
    for i in range(3):
        for t in (rep.out, rep.o, rep.dq, rep.dk, rep.dv):   # eager work between the replays
            t.fill_(float(i + 3))
        rep.lse.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((rep.out, rep.lse, rep.o, rep.dq), ref):
            assert torch.equal(got, want), f"replay {i}"
        assert torch.equal(rep.dk, ref_dk) and torch.equal(rep.dv, ref_dv), f"replay {i}"


# ---- the kernel forms the long shapes run.  The row-owning kernels (forward, dQ) exist with one, two
# and four key splits per workgroup; the automatic choice is four for every small shape, so the other
# two are forced through the descriptor here and must match the oracle on the full tensors.
@pytest.mark.parametrize("ks", [1, 2])
@pytest.mark.parametrize("hq,hkv,d,c,cp,w,rank", [
    (4, 1, 128, 200, 4, 2, 2),    # GQA 4:1: four heads stacked in a workgroup, ragged chunk
    (8, 1, 64, 96, 2, 1, 1),      # GQA 8:1, head_dim 64
    (6, 2, 128, 33, 3, 3, 1),     # group of 3: no stacking
    (2, 2, 128, 300, 2, 2, 0),    # more than one 256-row workgroup per half, ragged
    (4, 2, 64, 257, 2, 2, 1),
    (1, 1, 128, 520, 2, 2, 1),
])
def test_forced_key_splits_full_parity(ks, hq, hkv, d, c, cp, w, rank):
    cfg = RingConfig(f"ks{ks}_h{hq}_{hkv}_d{d}_c{c}_cp{cp}_r{rank}", cp=cp, w=w, rank=rank, hq=hq, hkv=hkv, d=d, c=c,
                     dtype="bf16", sigma=0.7, seed=500 + c + ks)
    inp = make_inputs(cfg)
    ref = oracle_full(cfg, inp)
    run = Replayed(cfg, inp, extra_flags=P.key_splits(ks))
    check_full(run.run(fuse_merge=True), ref)
    check_full(run.run(fuse_merge=False), ref)


@pytest.mark.parametrize("ks", [1, 2])
@pytest.mark.parametrize("idx", [2, 3, 4])
def test_forced_key_splits_on_shrunken_benchmark_configs(ks, idx):
    cfg = CONFIGS[idx].shrunk(320 if CONFIGS[idx].cp < 16 else 192).on_rank(CONFIGS[idx].cp // 2)
    inp = make_inputs(cfg)
    check_full(Replayed(cfg, inp, extra_flags=P.key_splits(ks)).run(), oracle_full(cfg, inp))


def test_shape_that_takes_one_and_two_key_splits_by_itself():
    """8192 local rows, two kv heads with four q heads each: the step that sees the early chunk only has
    256 workgroups of 4 heads x 64 rows (one key split), the diagonal step 512 of 4 x 32 rows (two key
    splits), both chosen by the library; the dK/dV kernel walks 4 heads x 128 query tiles per key tile."""
    cfg = RingConfig("natural_ks1_ks2", cp=2, w=2, rank=1, hq=8, hkv=2, d=128, c=4096, dtype="bf16", sigma=0.5, seed=4242)
    inp = make_inputs(cfg)
    check_full(Replayed(cfg, inp).run(), oracle_full(cfg, inp))


def test_one_chunk_pair_is_plain_causal_attention():
    """d_cp = 1 (Sec. "Comparison with DS-Ulysses & Megatron-CP": 2D-Attention with d_cp = 1 is Ulysses): the one
    rank holds the whole sequence in natural order and its single step is unchunked causal attention."""
    for hq, hkv, d, c in [(4, 2, 128, 333), (2, 1, 64, 500), (8, 8, 128, 160)]:
        cfg = RingConfig(f"cp1_h{hq}_{hkv}_d{d}_c{c}", cp=1, w=1, rank=0, hq=hq, hkv=hkv, d=d, c=c, dtype="bf16",
                         sigma=0.6, seed=900 + c)
        inp = make_inputs(cfg)
        pos = np.arange(cfg.S)
        assert np.array_equal(orc.zigzag_positions(1, 0, c), pos)
        dq, dk, dv, out, lse, delta = orc.attention_backward(inp["q"], inp["k_all"], inp["v_all"], inp["d_out"], pos, pos, cfg.scale)
        run = Replayed(cfg, inp).run()
        assert len(run.rep.plan) == 1 and run.rep.plan[0]["block_class"] == (P.DIAG, P.SKIP, P.FULL, P.DIAG)
        check_full(run, dict(out=out, lse=lse, dq=dq, dk=dk, dv=dv))


@pytest.mark.parametrize("hq,hkv,d,c,cp,w,rank,flags", [
    (4, 2, 128, 200, 4, 2, 1, 0),
    (4, 1, 64, 130, 2, 2, 1, 0),
    (2, 2, 128, 300, 2, 2, 0, 1 << 8),   # one key split
])
def test_causal_replay_with_batch_two(hq, hkv, d, c, cp, w, rank, flags):
    """Two sequences in one call (batch stride and batch x head indexing of all three matrix-core kernels on the
    causal path): each batch element must match the oracle of its own data."""
    cfgs = [RingConfig(f"batch2_{i}_h{hq}_{hkv}_d{d}_c{c}", cp=cp, w=w, rank=rank, hq=hq, hkv=hkv, d=d, c=c, dtype="bf16",
                       sigma=0.7, seed=600 + 10 * i + c) for i in range(2)]
    inps = [make_inputs(cf) for cf in cfgs]
    singles = [Replayed(cf, inp) for cf, inp in zip(cfgs, inps)]
    shape = ring.RingShape(cp=cp, w=w, rank=rank, hq=hq, hkv=hkv, d=d, c=c, dtype=P.BF16, scale=cfgs[0].scale, batch=2,
                           extra_flags=flags)
    rep = ring.RingReplay(shape, DEV)
    q = torch.cat([r.q for r in singles]).contiguous()
    d_o = torch.cat([r.d_o for r in singles]).contiguous()
    k_by_src = torch.cat([r.k_by_src for r in singles], dim=1).contiguous()
    v_by_src = torch.cat([r.v_by_src for r in singles], dim=1).contiguous()
    rep.forward(q, k_by_src, v_by_src)
    rep.backward(q, k_by_src, v_by_src, d_o)
    torch.cuda.synchronize()
    for i, (one, cf, inp) in enumerate(zip(singles, cfgs, inps)):
        # view batch element i through the single-sequence accessors
        one.rep.out, one.rep.lse, one.rep.o = rep.out[i:i + 1], rep.lse[i:i + 1], rep.o[i:i + 1]
        one.rep.dq, one.rep.dk, one.rep.dv = rep.dq[i:i + 1], rep.dk[:, i:i + 1], rep.dv[:, i:i + 1]
        check_full(one, oracle_full(cf, inp))


def test_rows_without_any_key_have_no_effect_on_the_backward():
    """A row whose softmax_lse is -inf saw no key in the whole attention: its probabilities are zero, so
    it must contribute nothing to dK/dV and get a zero dQ (no NaN from exp(+inf))."""
    b, hq, hkv, d, nq, nk = 1, 2, 1, 128, 200, 300
    rng = np.random.default_rng(5)
    mk = lambda *s: round_to_bf16(rng.standard_normal(s).astype(np.float32) * 0.5)
    q, do, k, v = mk(b, hq, nq, d), mk(b, hq, nq, d), mk(b, hkv, nk, d), mk(b, hkv, nk, d)
    scale = 1.0 / np.sqrt(d)
    blind = np.zeros(nq, bool)
    blind[[0, 63, 64, 130, 199]] = True
    ref = orc.attention_backward(q[0], k[0], v[0], do[0], np.zeros(nq, int), np.zeros(nk, int), scale, causal=False)
    lse = ref[4].copy()
    lse[:, blind] = -np.inf
    delta = ref[5].copy()
    delta[:, blind] = 0.0
    # the oracle of "these rows take no part": the same backward with the blind rows left out
    keep = ~blind
    dq_keep, dk_ref, dv_ref = orc.step_backward(q[0][:, keep], k[0], v[0], do[0][:, keep], lse[:, keep], delta[:, keep],
                                                np.zeros(keep.sum(), int), np.zeros(nk, int), scale, causal=False)
    dq_ref = np.zeros((hq, nq, d))
    dq_ref[:, keep] = dq_keep
    desc = P.make_desc(batch=b, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, q_len=nq, kv_len=nk, dtype=P.BF16, softmax_scale=scale)
    dq = torch.zeros(b, hq, nq, d, device=DEV)
    dk, dv = torch.empty(b, hkv, nk, d, device=DEV), torch.empty(b, hkv, nk, d, device=DEV)
    P.attn_step_bwd(desc, to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16"), None, to_dev(do, "bf16"),
                    torch.from_numpy(lse[None].astype(np.float32)).to(DEV), torch.from_numpy(delta[None].astype(np.float32)).to(DEV),
                    dq, dk, dv, workspace_for(desc))
    torch.cuda.synchronize()
    assert torch.isfinite(dq).all() and torch.isfinite(dk).all() and torch.isfinite(dv).all()
    assert max_abs(dq[0].cpu().numpy(), dq_ref) <= TOL_O and float(dq[0][:, torch.from_numpy(blind)].abs().max()) == 0.0
    assert max_abs(dk[0].cpu().numpy(), dk_ref) <= TOL_O and max_abs(dv[0].cpu().numpy(), dv_ref) <= TOL_O


# ------------------------------------------------------------------------------ direct calls, edge cases
def _direct(dtype, b, hq, hkv, d, nq, nk, seed, strided=False, accum=False):
    rng = np.random.default_rng(seed)
    mk = (lambda *s: round_to_bf16(rng.standard_normal(s).astype(np.float32) * 0.5)) if dtype == "bf16" else \
         (lambda *s: rng.standard_normal(s).astype(np.float32))
    q, do = mk(b, hq, nq, d), mk(b, hq, nq, d)
    k_buf, v_buf = mk(b, hkv, max(nk, 1), d), mk(b, hkv, max(nk, 1), d)   # never an empty allocation
    k, v = k_buf[:, :, :nk], v_buf[:, :, :nk]
    scale = 1.0 / np.sqrt(d)
    code = P.BF16 if dtype == "bf16" else P.FP32
    kw = {}
    if strided:   # token-major storage [b, token, head, d] viewed as [b, head, token, d]
        kw = dict(q_stride=(nq * hq * d, d, hq * d), kv_stride=(nk * hkv * d, d, hkv * d), o_stride=(nq * hq * d, d, hq * d))
    desc = P.make_desc(batch=b, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, q_len=nq, kv_len=nk, dtype=code,
                       softmax_scale=scale, **kw)

    def up(x, dt):
        t = to_dev(x, dt)
        return t.permute(0, 2, 1, 3).contiguous() if strided else t   # physical layout

    tq, tdo = up(q, dtype), up(do, dtype)
    tk, tv = (up(k, dtype), up(v, dtype)) if nk else (up(k_buf, dtype), up(v_buf, dtype))
    phys = (b, nq, hq, d) if strided else (b, hq, nq, d)
    out = torch.full(phys, 7.0, device=DEV)
    lse = torch.full((b, hq, nq), 7.0, device=DEV)
    P.attn_step_fwd(desc, tq, tk, tv, out, lse)
    torch.cuda.synchronize()
    got_out = (out.permute(0, 2, 1, 3) if strided else out).cpu().numpy()
    got_lse = lse.cpu().numpy()
    refs = [orc.attention_backward(q[i], k[i], v[i], do[i], np.zeros(nq, int), np.zeros(nk, int), scale, causal=False)
            for i in range(b)]
    ref_out = np.stack([r[3] for r in refs])
    ref_lse = np.stack([r[4] for r in refs])
    tol_o, tol_l = (TOL_O, TOL_LSE) if dtype == "bf16" else (2e-4, 1e-4)
    if nk == 0:
        assert np.all(got_out == 0) and np.all(np.isneginf(got_lse))
    else:
        assert max_abs(got_out, ref_out) <= tol_o and max_abs(got_lse, ref_lse) <= tol_l
    # backward from the oracle's exact row statistics
    o_store = up(ref_out.astype(np.float32), "fp32").to(torch.bfloat16 if dtype == "bf16" else torch.float32)
    lse_dev = torch.from_numpy(np.where(np.isfinite(ref_lse), ref_lse, -np.inf).astype(np.float32)).to(DEV)
    delta = torch.empty(b, hq, nq, device=DEV)
    dq = torch.zeros(phys, device=DEV)
    fill = 0.5 if accum else 9.0
    dk = torch.full((b, hkv, max(nk, 1), d), fill, device=DEV)   # one spare row when nk == 0: never a NULL pointer
    dv = torch.full((b, hkv, max(nk, 1), d), fill, device=DEV)
    desc.flags = P.COMPUTE_DELTA | (P.ACCUM_DKV if accum else 0)
    P.attn_step_bwd(desc, tq, tk, tv, o_store, tdo, lse_dev, delta, dq, dk, dv, workspace_for(desc))
    torch.cuda.synchronize()
    if nk > 0 and nq > 0:
        off = fill if accum else 0.0
        assert max_abs((dq.permute(0, 2, 1, 3) if strided else dq).cpu().numpy(), np.stack([r[0] for r in refs])) <= tol_o
        assert max_abs(dk.cpu().numpy() - off, np.stack([r[1] for r in refs])) <= tol_o
        assert max_abs(dv.cpu().numpy() - off, np.stack([r[2] for r in refs])) <= tol_o


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("nq,nk", [(333, 517), (1, 1), (64, 0), (70, 3), (5, 700)])
def test_non_causal_ragged_lengths(dtype, nq, nk):
    _direct(dtype, 2, 4, 2, 128 if dtype == "bf16" else 32, nq, nk, seed=nq + nk)


@pytest.mark.parametrize("hq,hkv,d,nq,nk", [(2, 2, 128, 1900, 200), (4, 1, 64, 1000, 130), (8, 8, 128, 700, 100)])
def test_few_key_tiles_many_query_tiles(hq, hkv, d, nq, nk):
    """Far fewer key tiles than CUs: several workgroups share a key tile's query loop, their number
    capped by the cost of the final summation (7, 10 and 4 here: uneven shares of the loop)."""
    _direct("bf16", 1, hq, hkv, d, nq, nk, seed=nq * 7 + nk)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_token_major_strides_and_accumulating_dkv(dtype):
    _direct(dtype, 2, 4, 2, 64, 130, 190, seed=3, strided=True, accum=True)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("fp32", 32)])
def test_one_sided_backward_flags_split_the_step_exactly(dtype, d):
    """dK/dV-only then dQ-only must reproduce the full call and leave the other side untouched."""
    b, hq, hkv, nq, nk = 1, 4, 2, 200, 330
    rng = np.random.default_rng(11)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    mk = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32) * 0.5).to(DEV).to(tdt)
    q, do, o = mk(b, hq, nq, d), mk(b, hq, nq, d), mk(b, hq, nq, d)
    k, v = mk(b, hkv, nk, d), mk(b, hkv, nk, d)
    lse = torch.from_numpy(rng.uniform(3.0, 5.0, (b, hq, nq)).astype(np.float32)).to(DEV)
    desc = P.make_desc(batch=b, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, q_len=nq, kv_len=nk,
                       dtype=P.BF16 if dtype == "bf16" else P.FP32, softmax_scale=1.0 / np.sqrt(d))
    res = []
    for split in (False, True):
        delta = torch.empty(b, hq, nq, device=DEV)
        dq = torch.full((b, hq, nq, d), 0.25, device=DEV)
        dk, dv = torch.full((b, hkv, nk, d), 9.0, device=DEV), torch.full((b, hkv, nk, d), 9.0, device=DEV)
        if not split:
            desc.flags = P.COMPUTE_DELTA
            P.attn_step_bwd(desc, q, k, v, o, do, lse, delta, dq, dk, dv, workspace_for(desc))
        else:
            desc.flags = P.COMPUTE_DELTA | P.BWD_ONLY_DKV
            P.attn_step_bwd(desc, q, k, v, o, do, lse, delta, None, dk, dv, workspace_for(desc))
            torch.cuda.synchronize()
            assert torch.all(dq == 0.25)
            keep = dk.clone()
            desc.flags = P.BWD_ONLY_DQ
            P.attn_step_bwd(desc, q, k, v, None, do, lse, delta, dq, None, None)
            torch.cuda.synchronize()
            assert torch.equal(dk, keep)
        torch.cuda.synchronize()
        res.append((dq.clone(), dk.clone(), dv.clone()))
    for a, c in zip(res[0], res[1]):                  # dq, dk, dv: every sum runs in a fixed order
        assert torch.equal(a, c)


def test_q_len_zero_is_a_noop():
    desc = P.make_desc(batch=1, n_q_heads=2, n_kv_heads=2, head_dim=128, q_len=0, kv_len=64, dtype=P.BF16, softmax_scale=0.1)
    x = torch.zeros(1, 2, 64, 128, dtype=torch.bfloat16, device=DEV)
    f = torch.zeros(1, 2, 64, 128, device=DEV)
    P.attn_step_fwd(desc, x, x, x, f, f)
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------ full benchmark sizes
@pytest.mark.parametrize("which_rank", ["first", "middle"])
def test_config2_full_size_full_tensor_parity(which_rank):
    """Rank 0 sees its own chunk and later ranks' (only its late half works); rank cp/2 also sees earlier ranks'
    chunks (all rows against the early keys: the step class in which the dK/dV query loops are shared)."""
    cfg = CONFIGS[1] if which_rank == "first" else CONFIGS[1].on_rank(CONFIGS[1].cp // 2)
    inp = make_inputs(cfg)
    run = Replayed(cfg, inp).run()
    check_full(run, oracle_full(cfg, inp))


def _edges(n, tiles=(16, 32, 64, 128, 256)):
    """Offsets at the ends of a run of n tokens and one either side of early and late tile edges."""
    e = {0, 1, n - 2, n - 1}
    for t in tiles:
        for k in (1, 3, n // t - 1):
            e.update({k * t - 1, k * t, k * t + 1})
    return {x for x in e if 0 <= x < n}


def _sample_rows(cfg, n_random, seed):
    c, L = cfg.c, cfg.L
    rows = {base + x for base in (0, c) for x in _edges(c)}
    rng = np.random.default_rng(seed)
    return np.array(sorted(rows | set(rng.integers(0, L, n_random).tolist())), dtype=np.int64)


def _sample_keys(cfg, n_random, seed):
    """Local key offsets inside a source rank's chunk pair: the ends of both halves, one either side of tile
    edges of 32, 64 and 128 keys near both ends of both halves, and seeded random ones."""
    c, L = cfg.c, cfg.L
    keys = {base + x for base in (0, c) for x in _edges(c, tiles=(32, 64, 128))}
    rng = np.random.default_rng(seed)
    return np.array(sorted(keys | set(rng.integers(0, L, n_random).tolist())), dtype=np.int64)


def _sources(cfg):
    """Source ranks whose dK/dV are checked key by key: the own chunk, the first and the last rank, and the
    neighbours in the ring either side (classes: earlier source, own chunk, later source)."""
    r, cp = cfg.rank, cfg.cp
    return sorted({0, r // 2, (r - 1) % cp, r, (r + 1) % cp, cp - 1})


@pytest.mark.parametrize("which_rank", ["first", "middle"])
@pytest.mark.parametrize("idx,n_random", [(2, 24), (3, 16), (4, 8)])
def test_full_size_sampled_rows_sampled_keys_and_gradient_identities(idx, n_random, which_rank):
    """The benchmark shapes a full fp64 backward is out of reach for (8 to 123 TFLOP): exact fp64 O, LSE, dQ of
    sampled rows over ALL keys; exact fp64 dK_j, dV_j of sampled keys j of several source ranks over all local
    rows (the definition dK_j = scale sum_h sum_i dS_ij q_i, dV_j = sum_h sum_i P_ij dO_i restricted to those
    keys, with the device's LSE and delta, which the sampled rows validate); and the three sum identities."""
    cfg = CONFIGS[idx] if which_rank == "first" else CONFIGS[idx].on_rank(CONFIGS[idx].cp // 2)
    inp = make_inputs(cfg)
    run = Replayed(cfg, inp).run()
    rows = _sample_rows(cfg, n_random, seed=idx)
    pos_all = orc.zigzag_positions(cfg.cp, cfg.rank, cfg.c)
    pos_q = pos_all[rows]
    # exact rows: O, LSE and dQ of the sampled rows over all S keys
    errs = {"out": 0.0, "lse": 0.0, "dq": 0.0, "delta": 0.0}
    got_out, got_lse, got_dq = run.out(), run.lse(), run.dq()
    got_delta = run.rep.delta[0].double().cpu().numpy()
    g = cfg.hq // cfg.hkv
    for h in range(cfg.hq):
        sl = slice(h // g, h // g + 1)
        dq, _, _, out, lse, delta = orc.attention_backward(inp["q"][h:h + 1, rows], inp["k_all"][sl], inp["v_all"][sl],
                                                           inp["d_out"][h:h + 1, rows], pos_q, np.arange(cfg.S), cfg.scale)
        errs["out"] = max(errs["out"], max_abs(got_out[h, rows], out[0]))
        errs["lse"] = max(errs["lse"], max_abs(got_lse[h, rows], lse[0]))
        errs["dq"] = max(errs["dq"], max_abs(got_dq[h, rows], dq[0]))
        errs["delta"] = max(errs["delta"], max_abs(got_delta[h, rows], delta[0]))
    print(f"[sampled rows] {cfg.name}: {errs} rows={len(rows)}", flush=True)
    assert errs["out"] <= TOL_O and errs["dq"] <= TOL_O and errs["lse"] <= TOL_LSE and errs["delta"] <= TOL_O
    # exact keys: dK_j, dV_j of sampled keys of several sources, over all local rows and all heads of the group
    keys = _sample_keys(cfg, 3 * n_random, seed=100 + idx)
    kerr = {"dk": 0.0, "dv": 0.0}
    classes = set()
    n_keys = 0
    for src in _sources(cfg):
        classes.add("earlier" if src < cfg.rank else "own" if src == cfg.rank else "later")
        pos_k = orc.zigzag_positions(cfg.cp, src, cfg.c)[keys]
        _, dk, dv = orc.step_backward(inp["q"], inp["k_all"][:, pos_k], inp["v_all"][:, pos_k], inp["d_out"], got_lse, got_delta,
                                      pos_all, pos_k, cfg.scale)
        idx_t = torch.from_numpy(keys).to(DEV)
        kerr["dk"] = max(kerr["dk"], max_abs(run.rep.dk[src, 0].index_select(1, idx_t).double().cpu().numpy(), dk))
        kerr["dv"] = max(kerr["dv"], max_abs(run.rep.dv[src, 0].index_select(1, idx_t).double().cpu().numpy(), dv))
        n_keys += len(keys)
    print(f"[sampled keys] {cfg.name}: {kerr} keys per kv head={n_keys} source classes={sorted(classes)}", flush=True)
    assert kerr["dk"] <= TOL_O and kerr["dv"] <= TOL_O
    assert classes == ({"own", "later"} if cfg.rank == 0 else {"earlier", "own", "later"})
    # identities that hold at any size, on the device results
    dk = run.rep.dk.double().sum(dim=(0, 1, 3)).cpu().numpy()          # [hkv, d]: sum over all keys
    dv = run.rep.dv.double().sum(dim=(0, 1, 3)).cpu().numpy()
    dk_mass = run.rep.dk.double().abs().sum(dim=(0, 1, 3)).cpu().numpy()
    dv_mass = run.rep.dv.double().abs().sum(dim=(0, 1, 3)).cpu().numpy()
    do_sum = inp["d_out"].astype(np.float64).reshape(cfg.hkv, g, cfg.L, cfg.d).sum(axis=(1, 2))
    r_dk = np.abs(dk).max() / dk_mass.max()
    r_dv = np.abs(dv - do_sum).max() / dv_mass.max()
    qdq = float((run.rep.dq[0].double().cpu().numpy() * inp["q"]).sum())
    kdk = 0.0
    for s in range(cfg.cp):
        pos = orc.zigzag_positions(cfg.cp, s, cfg.c)
        kdk += float((run.rep.dk[s, 0].double().cpu().numpy() * inp["k_all"][:, pos]).sum())
    scale_qk = float(np.abs(run.rep.dq[0].double().cpu().numpy() * inp["q"]).sum())
    r_qk = abs(qdq - kdk) / scale_qk
    print(f"[identities] {cfg.name}: sum dK {r_dk:.2e}  sum dV {r_dv:.2e}  <q,dQ>-<k,dK> {r_qk:.2e}", flush=True)
    assert r_dk < 2e-3 and r_dv < 2e-3 and r_qk < 2e-3
    if idx == 3 and which_rank == "first":   # double ring vs plain ring: same result up to the rounding of P
        lin = Replayed(RingConfig(**{**cfg.__dict__, "w": cfg.cp}), inp).run()
        assert max_abs(lin.out(), got_out) < 1e-3 and max_abs(lin.lse(), got_lse) < 1e-4
        assert float((lin.rep.dk - run.rep.dk).abs().max()) < 2e-3
        assert float((lin.rep.dv - run.rep.dv).abs().max()) < 2e-3
