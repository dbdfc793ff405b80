"""Pins of the layout oracle: element-by-element definitions in plain loops on tiny shapes, round trips, adjointness."""
import numpy as np

from oracle import layout_oracle as lo


def test_pack_heads_and_unpack_tokens_by_plain_loops():
    rng = np.random.default_rng(0)
    s, H, d, d_hp = 3, 4, 2, 2
    hl = H // d_hp
    x = rng.standard_normal((s, H, d))
    m = lo.seq_a2a_pack_heads(x, d_hp)
    for j in range(d_hp):
        for h in range(hl):
            for t in range(s):
                assert np.array_equal(m[j, h, t], x[t, j * hl + h])
    # a GPU receives message i from GPU i: its own head group, that GPU's tokens
    per_gpu = [rng.standard_normal((s, H, d)) for _ in range(d_hp)]
    me = 1
    recv = np.stack([lo.seq_a2a_pack_heads(per_gpu[i], d_hp)[me] for i in range(d_hp)])
    u = lo.seq_a2a_unpack_tokens(recv)
    for h in range(hl):
        for i in range(d_hp):
            for t in range(s):
                assert np.array_equal(u[h, i * s + t], per_gpu[i][t, me * hl + h])


def test_second_all_to_all_is_the_inverse_of_the_first():
    rng = np.random.default_rng(1)
    s, H, d, d_hp = 5, 8, 4, 4
    per_gpu = [rng.standard_normal((s, H, d)) for _ in range(d_hp)]
    sent = [lo.seq_a2a_pack_heads(x, d_hp) for x in per_gpu]
    local = [lo.seq_a2a_unpack_tokens(np.stack([sent[i][j] for i in range(d_hp)])) for j in range(d_hp)]
    back_sent = [lo.seq_a2a_pack_tokens(x, d_hp) for x in local]
    for i in range(d_hp):
        got = lo.seq_a2a_unpack_heads(np.stack([back_sent[j][i] for j in range(d_hp)]))
        assert np.array_equal(got, per_gpu[i])


def test_replication_and_its_gradient_are_adjoint():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((3, 4, 2)).astype(np.float32)
    g = rng.standard_normal((6, 4, 2)).astype(np.float32)
    r = lo.replicate_kv(x, 2)
    assert r.shape == (6, 4, 2) and np.array_equal(r[2], x[1]) and np.array_equal(r[3], x[1])
    # <replicate(x), g> == <x, reduce(g)>
    lhs = float((r.astype(np.float64) * g).sum())
    rhs = float((x.astype(np.float64) * lo.reduce_replicas(g, 2)).sum())
    assert abs(lhs - rhs) < 1e-4
    assert np.array_equal(lo.reduce_replicas(g, 1), g)
