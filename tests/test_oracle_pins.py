"""Pins of the fp64 oracle to things other than itself: brute force, closed forms,
library routines, finite differences and counting arguments.  CPU only."""
import itertools
import math

import numpy as np
import pytest
import torch

import oracle as orc


def _rand(shape, seed, sigma=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * sigma


def _case(hq=4, hkv=2, cp=2, rank=1, c=3, d=5, seed=0):
    s = 2 * cp * c
    q = _rand((hq, 2 * c, d), seed)
    do = _rand((hq, 2 * c, d), seed + 1)
    k = _rand((hkv, s, d), seed + 2)
    v = _rand((hkv, s, d), seed + 3)
    pos_q = orc.zigzag_positions(cp, rank, c)
    pos_k = np.arange(s)
    return q, k, v, do, pos_q, pos_k


# ------------------------------------------------------------------ forward: brute force
def _brute_forward(q, k, v, pos_q, pos_k, scale, causal=True):
    hq, lq, d = q.shape
    g = hq // k.shape[0]
    out = np.zeros((hq, lq, d))
    lse = np.full((hq, lq), -math.inf)
    for h in range(hq):
        for i in range(lq):
            w = []
            for j in range(k.shape[1]):
                if causal and pos_k[j] > pos_q[i]:
                    continue
                sc = 0.0
                for t in range(d):
                    sc += q[h, i, t] * k[h // g, j, t]
                w.append((j, math.exp(scale * sc)))
            z = sum(x for _, x in w)
            if z == 0.0:
                continue
            lse[h, i] = math.log(z)
            for j, x in w:
                for t in range(d):
                    out[h, i, t] += x / z * v[h // g, j, t]
    return out, lse


@pytest.mark.parametrize("hq,hkv,cp,rank", [(4, 2, 2, 1), (2, 2, 3, 0), (3, 1, 2, 0)])
def test_forward_matches_triple_loop(hq, hkv, cp, rank):
    q, k, v, _, pos_q, pos_k = _case(hq, hkv, cp, rank)
    out, lse = orc.attention_forward(q, k, v, pos_q, pos_k, 0.37)
    bo, bl = _brute_forward(q, k, v, pos_q, pos_k, 0.37)
    np.testing.assert_allclose(out, bo, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, bl, rtol=0, atol=1e-13)


def test_chunk_partial_matches_triple_loop_with_blind_rows():
    # rank 0 against the chunk of rank 1: the low half of Q sees nothing
    cp, c = 2, 3
    q, k, v, _, pos_q, _ = _case(2, 1, cp, 0, c)
    pos_k = orc.zigzag_positions(cp, 1, c)
    kc, vc = k[:, pos_k], v[:, pos_k]
    out, lse = orc.attention_forward(q, kc, vc, pos_q, pos_k, 0.5)
    bo, bl = _brute_forward(q, kc, vc, pos_q, pos_k, 0.5)
    np.testing.assert_allclose(out, bo, atol=1e-13)
    assert np.all(np.isneginf(lse[:, :c])) and np.all(out[:, :c] == 0)
    np.testing.assert_allclose(lse[:, c:], bl[:, c:], atol=1e-13)


# ------------------------------------------------------------------ forward: closed forms
def test_zero_queries_give_running_mean_and_log_count():
    q, k, v, _, pos_q, pos_k = _case(2, 1, 3, 1, 4)
    out, lse = orc.attention_forward(np.zeros_like(q), k, v, pos_q, pos_k, 0.3)
    np.testing.assert_allclose(lse, np.broadcast_to(np.log(pos_q + 1.0), lse.shape), atol=1e-13)
    run_mean = np.cumsum(v[0], axis=0) / (np.arange(v.shape[1]) + 1.0)[:, None]
    np.testing.assert_allclose(out[1], run_mean[pos_q], atol=1e-13)


def test_first_token_row():
    q, k, v, _, pos_q, pos_k = _case(2, 2, 2, 0, 3)
    assert pos_q[0] == 0
    out, lse = orc.attention_forward(q, k, v, pos_q, pos_k, 0.25)
    for h in range(2):
        np.testing.assert_allclose(out[h, 0], v[h, 0], atol=1e-14)
        np.testing.assert_allclose(lse[h, 0], 0.25 * q[h, 0] @ k[h, 0], atol=1e-14)


def test_constant_values_and_row_stochastic():
    q, k, v, _, pos_q, pos_k = _case()
    row = np.arange(v.shape[2], dtype=np.float64) - 1.5
    out, _ = orc.attention_forward(q, k, np.broadcast_to(row, v.shape), pos_q, pos_k, 1.1)
    np.testing.assert_allclose(out, np.broadcast_to(row, out.shape), atol=1e-13)
    out1, _ = orc.attention_forward(q, k, np.ones_like(v), pos_q, pos_k, 1.1)
    np.testing.assert_allclose(out1, 1.0, atol=1e-13)


def test_future_keys_have_no_effect_bitwise():
    q, k, v, _, pos_q, pos_k = _case(2, 1, 2, 0, 4)
    out, lse = orc.attention_forward(q, k, v, pos_q, pos_k, 0.4)
    k2, v2 = k.copy(), v.copy()
    cut = int(pos_q[3])  # row 3 must not see anything after its own position
    k2[:, cut + 1:] += 100.0
    v2[:, cut + 1:] -= 50.0
    out2, lse2 = orc.attention_forward(q, k2, v2, pos_q, pos_k, 0.4)
    assert np.array_equal(out[:, :4], out2[:, :4]) and np.array_equal(lse[:, :4], lse2[:, :4])
    assert not np.array_equal(out[:, 4:], out2[:, 4:])


# ------------------------------------------------------------------ forward: library routines
def test_non_causal_is_library_softmax_matmul():
    q, k, v, _, pos_q, pos_k = _case(2, 2, 1, 0, 6, d=7)
    out, lse = orc.attention_forward(q, k, v, pos_q, pos_k, 0.61, causal=False)
    tq, tk, tv = map(torch.from_numpy, (q, k, v))
    s = 0.61 * tq @ tk.transpose(1, 2)
    np.testing.assert_allclose(out, (torch.softmax(s, -1) @ tv).numpy(), atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), atol=1e-13)


def _torch_causal(q, k, v, pos_q, pos_k, scale):
    g = q.shape[0] // k.shape[0]
    tq = torch.tensor(q, requires_grad=True)
    tk = torch.tensor(k, requires_grad=True)
    tv = torch.tensor(v, requires_grad=True)
    mask = torch.from_numpy(pos_k[None, :] <= pos_q[:, None])
    o = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk.repeat_interleave(g, 0)[None], tv.repeat_interleave(g, 0)[None],
        attn_mask=mask, scale=scale)[0]
    return tq, tk, tv, o


def test_causal_gqa_is_library_sdpa_forward_and_autograd():
    q, k, v, do, pos_q, pos_k = _case(4, 2, 3, 2, 4, d=8)
    tq, tk, tv, o = _torch_causal(q, k, v, pos_q, pos_k, 0.3)
    (o * torch.from_numpy(do)).sum().backward()
    dq, dk, dv, out, _, _ = orc.attention_backward(q, k, v, do, pos_q, pos_k, 0.3)
    np.testing.assert_allclose(out, o.detach().numpy(), atol=1e-13)
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-13)


# ------------------------------------------------------------------ backward: finite differences
def test_backward_matches_central_differences():
    q, k, v, do, pos_q, pos_k = _case(2, 1, 2, 1, 2, d=3, seed=5)
    scale = 0.7
    dq, dk, dv, *_ = orc.attention_backward(q, k, v, do, pos_q, pos_k, scale)

    def loss(q_, k_, v_):
        return float((orc.attention_forward(q_, k_, v_, pos_q, pos_k, scale)[0] * do).sum())

    eps = 1e-5
    for arr, grad, which in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        num = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            args = [q.copy(), k.copy(), v.copy()]
            args[which][idx] += eps
            up = loss(*args)
            args[which][idx] -= 2 * eps
            num[idx] = (up - loss(*args)) / (2 * eps)
        np.testing.assert_allclose(grad, num, rtol=1e-6, atol=1e-8)


def test_gradient_sum_identities():
    q, k, v, do, pos_q, pos_k = _case(4, 2, 3, 1, 5, d=6, seed=9)
    dq, dk, dv, *_ = orc.attention_backward(q, k, v, do, pos_q, pos_k, 0.45)
    # scores enter only through q.k, so <q_i, dQ_i> summed equals <k_j, dK_j> summed
    np.testing.assert_allclose((q * dq).sum(), (k * dk).sum(), atol=1e-12)
    # softmax rows sum to one, every row sees a key: sum_j dV_j = sum_i dO_i per kv head
    g = q.shape[0] // k.shape[0]
    np.testing.assert_allclose(dv.sum(axis=1), do.reshape(k.shape[0], g, *do.shape[1:]).sum(axis=(1, 2)), atol=1e-12)
    # adding one vector u to every key shifts each row's scores by a constant, which
    # softmax ignores: d/dt loss(k + t u) = <u, sum_j dK_j> = 0 for every u
    np.testing.assert_allclose(dk.sum(axis=1), 0.0, atol=1e-12)


def test_steps_sum_to_global_backward():
    cp, c, rank = 4, 3, 2
    q, k, v, do, pos_q, pos_k = _case(4, 2, cp, rank, c, d=4, seed=11)
    dq, dk, dv, out, lse, delta = orc.attention_backward(q, k, v, do, pos_q, pos_k, 0.5)
    dq_sum = np.zeros_like(dq)
    dk_all = np.zeros_like(dk)
    dv_all = np.zeros_like(dv)
    for src in orc.double_ring_sources(cp, 2, rank):
        pk = orc.zigzag_positions(cp, src, c)
        a, b, cc = orc.step_backward(q, k[:, pk], v[:, pk], do, lse, delta, pos_q, pk, 0.5)
        dq_sum += a
        dk_all[:, pk] += b
        dv_all[:, pk] += cc
    np.testing.assert_allclose(dq_sum, dq, atol=1e-13)
    np.testing.assert_allclose(dk_all, dk, atol=1e-13)
    np.testing.assert_allclose(dv_all, dv, atol=1e-13)


# ------------------------------------------------------------------ Update / merge
def test_update_is_logsumexp_of_two_terms():
    from scipy.special import logsumexp
    a, b = _rand((3, 7), 1, 3.0), _rand((3, 7), 2, 3.0)
    oa, ob = _rand((3, 7, 4), 3), _rand((3, 7, 4), 4)
    out, lse = orc.update(oa, a, ob, b)
    np.testing.assert_allclose(lse, logsumexp(np.stack([a, b]), axis=0), atol=1e-14)
    wa = np.exp(a) / (np.exp(a) + np.exp(b))
    np.testing.assert_allclose(out, wa[..., None] * oa + (1 - wa)[..., None] * ob, atol=1e-14)


def test_update_neutral_element_and_equal_partials():
    a = _rand((2, 5), 1)
    oa = _rand((2, 5, 3), 2)
    ninf = np.full_like(a, -np.inf)
    for out, lse in (orc.update(oa, a, np.zeros_like(oa), ninf), orc.update(np.zeros_like(oa), ninf, oa, a)):
        assert np.array_equal(out, oa) and np.array_equal(lse, a)
    out, lse = orc.update(np.zeros_like(oa), ninf, np.zeros_like(oa), ninf)
    assert np.all(np.isneginf(lse)) and np.all(out == 0)
    out, lse = orc.update(oa, a, oa, a)
    np.testing.assert_allclose(lse, a + math.log(2.0), atol=1e-15)
    np.testing.assert_allclose(out, oa, atol=1e-15)


@pytest.mark.parametrize("rank", [0, 1, 3])
def test_merge_of_chunk_partials_is_unchunked_attention_in_any_order(rank):
    cp, c = 4, 3
    q, k, v, _, pos_q, pos_k = _case(4, 2, cp, rank, c, d=4, seed=21)
    ref_out, ref_lse = orc.attention_forward(q, k, v, pos_q, pos_k, 0.9)
    parts = []
    for src in range(cp):
        pk = orc.zigzag_positions(cp, src, c)
        parts.append(orc.attention_forward(q, k[:, pk], v[:, pk], pos_q, pk, 0.9))
    for order in itertools.permutations(range(cp)):
        out, lse = orc.merge_partials(parts, order)
        np.testing.assert_allclose(out, ref_out, atol=1e-12)
        np.testing.assert_allclose(lse, ref_lse, atol=1e-12)


# ------------------------------------------------------------------ layout, order, mask coverage
def test_zigzag_layout_of_first_benchmark_case():
    # first benchmark case: 8 chunks for 4 devices, device 0 holds chunks 0 and 7
    assert orc.zigzag_chunk_ids(4, 0) == (0, 7)
    pos = orc.zigzag_positions(4, 0, 128)
    assert pos[0] == 0 and pos[127] == 127 and pos[128] == 7 * 128 and pos[-1] == 1023
    # every position of the sequence is owned exactly once
    allpos = np.concatenate([orc.zigzag_positions(4, r, 128) for r in range(4)])
    assert np.array_equal(np.sort(allpos), np.arange(1024))


@pytest.mark.parametrize("cp,w", [(4, 1), (4, 2), (4, 4), (8, 4), (8, 2), (16, 4), (6, 3)])
def test_visit_order_properties(cp, w):
    for r in range(cp):
        order = orc.double_ring_sources(cp, w, r)
        assert order[0] == r and sorted(order) == list(range(cp))
        if w in (1, cp):
            assert order == [(r - t) % cp for t in range(cp)]
        # inside one outer step the sources stay inside one inner ring's ranks
        for a in range(cp // w):
            assert len({s // w for s in order[a * w:(a + 1) * w]}) == 1


@pytest.mark.parametrize("cp,c,w", [(4, 3, 1), (4, 3, 2), (4, 3, 4), (8, 2, 4), (8, 2, 2), (16, 1, 4)])
def test_quadrant_rule_covers_causal_mask_exactly_once(cp, c, w):
    s_total = 2 * cp * c
    ell = 2 * c
    for r in range(cp):
        pos_q = orc.zigzag_positions(cp, r, c)
        cover = np.zeros((ell, s_total), dtype=np.int64)
        for src in orc.double_ring_sources(cp, w, r):
            pk = orc.zigzag_positions(cp, src, c)
            cls = orc.quadrant_classes(orc.zigzag_chunk_ids(cp, r), orc.zigzag_chunk_ids(cp, src))
            block = np.zeros((ell, ell), dtype=bool)
            for a in range(2):
                for b in range(2):
                    sub = block[a * c:(a + 1) * c, b * c:(b + 1) * c]
                    if cls[a, b] == orc.FULL:
                        sub[:] = True
                    elif cls[a, b] == orc.DIAG:
                        sub[:] = np.tril(np.ones((c, c), dtype=bool))
            assert np.array_equal(block, pk[None, :] <= pos_q[:, None])
            n = int(block.sum())
            assert n == orc.step_pair_count(cp, r, src, c)
            assert n == (ell * (ell + 1) // 2 if src == r else ell * ell // 2)
            cover[:, pk] += block
        assert np.array_equal(cover, (np.arange(s_total)[None, :] <= pos_q[:, None]).astype(np.int64))


def test_total_pairs_of_the_benchmark_shapes():
    # pairs per head over all steps: L(L+1)/2 on the own chunk, L^2/2 on the others
    for cp, ell, want in ((4, 256, 131200), (8, 4096, 67110912), (8, 16384, 1073750016)):
        assert ell * (ell + 1) // 2 + (cp - 1) * ell * ell // 2 == want
