"""Plain fp64 oracle for the per-device ring-step attention of Double-Ring-Attention.

TEST INFRASTRUCTURE ONLY.  Slow, unblocked, written from the definitions; it shares
no code with the HIP path and must never be imported by it.  Everything is numpy
fp64; a matmul, exp and log are the only library primitives used.

What the method computes (paper: Sec. 2 "LLM Architecture with MHA/GQA" for the head
layout, Sec. 2 "Distributed Attention" for chunk-wise iteration over K/V and the
load-balanced causal reorder, Alg. 2 for the per-micro-step ``Attention`` + ``Update``
and the inner/outer ring order, Sec. 3.1 for the backward that circulates K/V together
with their gradients, Sec. "Selective Checkpoint++" for what the backward may consume:
the stored attention output and softmax_lse):

the ring with its merge is a re-association of the sums of ordinary causal softmax
attention, so the oracle of the whole replay is that definition written out over the
global sequence (``attention_forward`` / ``attention_backward``); the oracle of a single
micro-step is the same definition restricted to the visiting chunk's keys
(``attention_forward`` on the chunk, ``step_backward``), and the oracle of ``Update`` is
the two-term log-sum-exp combination (``update``).

Readings taken where the paper is silent (each is listed in the design notes):
  * Update formula, zigzag layout (2*cp chunks, rank r owns r and 2cp-1-r), ring
    direction (step t holds source (r-t) mod cp), W_{i,j} <-> rank = i*w + j,
    natural-log LSE, GQA mapping q head h -> kv head h // G, rows that see no key in
    a step give (0, -inf).

Pins (tests/test_oracle_pins.py): triple-loop brute force, closed forms (zero queries,
first token, constant values), row-stochasticity, exact causality, library softmax /
autograd special cases, central finite differences, gradient sum identities, merge
order invariance, exhaustive mask-coverage counts.  The double-ring visit order beyond
the text of Alg. 2 has no printed example to compare with (the figure is not
available): that ordering is "parity unpinned"; what is pinned is that it is a
permutation starting at the own chunk, reduces to the plain ring for w in {1, cp}, and
that the merged result does not depend on it.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "zigzag_chunk_ids", "zigzag_positions", "double_ring_sources", "quadrant_classes",
    "step_pair_count", "attention_forward", "attention_backward", "step_backward",
    "update", "merge_partials", "rowsum_delta", "SKIP", "FULL", "DIAG",
]

SKIP, FULL, DIAG = 0, 1, 2


# --------------------------------------------------------------------------------------
# Layout and visit order
# --------------------------------------------------------------------------------------
def zigzag_chunk_ids(cp: int, rank: int) -> tuple[int, int]:
    """Global chunk ids held by `rank` when the sequence is cut into 2*cp chunks and
    reordered for causal load balance (Sec. 2 "Distributed Attention", load-balanced
    Ring-Attention): one chunk from the front and its mirror from the back."""
    assert 0 <= rank < cp
    return rank, 2 * cp - 1 - rank


def zigzag_positions(cp: int, rank: int, c: int) -> np.ndarray:
    """Global token position of each of the 2c local rows of `rank` (low chunk first)."""
    lo, hi = zigzag_chunk_ids(cp, rank)
    return np.concatenate([lo * c + np.arange(c), hi * c + np.arange(c)]).astype(np.int64)


def double_ring_sources(cp: int, w: int, rank: int) -> list[int]:
    """Source rank whose K/V chunk `rank` holds at each micro-step of Alg. 2.

    GPUs W_{i,j} (i: which inner ring, j: place inside it) are numbered rank = i*w + j.
    Every send goes to the next rank of its ring and every receive comes from the
    previous one, so after `a` outer steps and `b` inner micro-steps the chunk in hand
    started at W_{i-a, j-b} (indices modulo cp/w and w).  Outer loop outermost.
    """
    assert cp % w == 0 and 0 <= rank < cp
    n_outer = cp // w
    i, j = divmod(rank, w)
    order = []
    for a in range(n_outer):
        for b in range(w):
            order.append(((i - a) % n_outer) * w + ((j - b) % w))
    return order


def quadrant_classes(q_ids, kv_ids) -> np.ndarray:
    """Class of each (q half, k half) block of a micro-step from the chunk ids alone:
    an earlier key chunk is fully visible, the same chunk is lower-triangular, a later
    one is invisible (causal mask, Fig. 2 caption: 1 or 0 per block)."""
    out = np.zeros((2, 2), dtype=np.int64)
    for a in range(2):
        for b in range(2):
            out[a, b] = FULL if kv_ids[b] < q_ids[a] else DIAG if kv_ids[b] == q_ids[a] else SKIP
    return out


def step_pair_count(cp: int, rank: int, src: int, c: int) -> int:
    """Number of (query, key) pairs with key position <= query position in one step,
    counted pair by pair from the positions (no shortcut)."""
    pq = zigzag_positions(cp, rank, c)
    pk = zigzag_positions(cp, src, c)
    return int((pk[None, :] <= pq[:, None]).sum())


# --------------------------------------------------------------------------------------
# The definition: masked softmax attention and its gradient
# --------------------------------------------------------------------------------------
def _allowed(pos_q, pos_k, causal):
    if causal:
        return pos_k[None, :] <= pos_q[:, None]
    return np.ones((len(pos_q), len(pos_k)), dtype=bool)


def attention_forward(q, k, v, pos_q, pos_k, scale, causal=True):
    """O and natural-log LSE of softmax(scale * q k^T + mask) v over the keys given.

    q: [Hq, Lq, d]; k, v: [Hkv, Lk, d]; q head h uses kv head h // (Hq // Hkv).
    Key j is visible to row i iff pos_k[j] <= pos_q[i] (or always when not causal).
    A row that sees no key returns O = 0 and LSE = -inf.
    With all S keys this is the whole-replay result; with one chunk's keys it is the
    `Attention(Q, K, V)` of one micro-step (Alg. 2).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    hq, lq, d = q.shape
    hkv = k.shape[0]
    g = hq // hkv
    assert hq == g * hkv
    ok = _allowed(np.asarray(pos_q), np.asarray(pos_k), causal)
    out = np.zeros((hq, lq, d))
    lse = np.full((hq, lq), -np.inf)
    seen = ok.any(axis=1)
    for h in range(hq):
        s = scale * (q[h] @ k[h // g].T)
        s = np.where(ok, s, -np.inf)
        m = np.where(seen, s.max(axis=1, initial=-np.inf), 0.0)
        e = np.exp(s - m[:, None])
        z = e.sum(axis=1)
        with np.errstate(divide="ignore"):
            lse[h] = np.where(seen, m + np.log(z), -np.inf)
        p = e / np.where(seen, z, 1.0)[:, None]
        out[h] = p @ v[h // g]
    return out, lse


def rowsum_delta(d_out, out):
    """D_i = sum_k dO_ik * O_ik, the per-row term of the softmax gradient."""
    return (np.asarray(d_out, np.float64) * np.asarray(out, np.float64)).sum(axis=-1)


def step_backward(q, k, v, d_out, lse, delta, pos_q, pos_k, scale, causal=True):
    """Gradient contributions of one key set, given the FINAL row statistics.

    lse [Hq, Lq] and delta [Hq, Lq] are those of the complete attention (all chunks
    merged); k, v are the visiting chunk (or all keys).  Returns
      dq  [Hq, Lq, d]  : this key set's share of dQ,
      dk, dv [Hkv, Lk, d]: gradient of these keys/values from this device's rows,
                           summed over the q heads that share the kv head.
    P_ij = exp(s_ij - LSE_i); dP = dO v^T; dS = P * (dP - D); dQ = scale dS k;
    dK = scale dS^T q; dV = P^T dO.
    """
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    d_out = np.asarray(d_out, np.float64)
    hq, lq, d = q.shape
    hkv = k.shape[0]
    g = hq // hkv
    ok = _allowed(np.asarray(pos_q), np.asarray(pos_k), causal)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for h in range(hq):
        kh = h // g
        s = scale * (q[h] @ k[kh].T)
        row_lse = np.where(np.isfinite(lse[h]), lse[h], 0.0)
        p = np.where(ok, np.exp(np.where(ok, s, 0.0) - row_lse[:, None]), 0.0)
        dp = d_out[h] @ v[kh].T
        ds = p * (dp - np.asarray(delta[h], np.float64)[:, None])
        dq[h] = scale * (ds @ k[kh])
        dk[kh] += scale * (ds.T @ q[h])
        dv[kh] += p.T @ d_out[h]
    return dq, dk, dv


def attention_backward(q, k, v, d_out, pos_q, pos_k, scale, causal=True):
    """dQ, dK, dV of <dO, O> for the complete attention over the keys given.
    Also returns (O, LSE, D) so callers can reuse them."""
    out, lse = attention_forward(q, k, v, pos_q, pos_k, scale, causal)
    delta = rowsum_delta(d_out, out)
    dq, dk, dv = step_backward(q, k, v, d_out, lse, delta, pos_q, pos_k, scale, causal)
    return dq, dk, dv, out, lse, delta


# --------------------------------------------------------------------------------------
# Update: merging a partial result into the running one (Alg. 2, the Update call)
# --------------------------------------------------------------------------------------
def update(out, lse, block_out, block_lse):
    """Combine two normalised partial attentions over disjoint key sets.

    lse' = log(exp(lse) + exp(block_lse));
    out' = exp(lse - lse') * out + exp(block_lse - lse') * block_out.
    A side with lse = -inf contributes nothing; (0, -inf) is the neutral element.
    Returns new arrays (inputs untouched).
    """
    out = np.asarray(out, np.float64)
    lse = np.asarray(lse, np.float64)
    block_out = np.asarray(block_out, np.float64)
    block_lse = np.asarray(block_lse, np.float64)
    hi = np.maximum(lse, block_lse)
    safe = np.where(np.isfinite(hi), hi, 0.0)
    wa = np.exp(lse - safe)
    wb = np.exp(block_lse - safe)
    tot = wa + wb
    with np.errstate(divide="ignore"):
        new_lse = np.where(np.isfinite(hi), safe + np.log(tot), -np.inf)
    den = np.where(tot > 0, tot, 1.0)
    new_out = (wa / den)[..., None] * out + (wb / den)[..., None] * block_out
    return new_out, new_lse


def merge_partials(partials, order=None):
    """Fold a list of (block_out, block_lse) into (0, -inf) with `update`, visiting
    them in `order` (default: list order)."""
    if order is None:
        order = range(len(partials))
    first = partials[0]
    out = np.zeros_like(np.asarray(first[0], np.float64))
    lse = np.full(np.asarray(first[1]).shape, -np.inf)
    for idx in order:
        out, lse = update(out, lse, partials[idx][0], partials[idx][1])
    return out, lse
