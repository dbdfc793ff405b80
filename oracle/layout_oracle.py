"""Plain oracle of the on-device layout steps either side of the ring (Alg. 1): the local
re-arrangements of SeqAlltoAll and the KV replication of GQA with its gradient reduction
(Sec. "KV Replication for GQA").

TEST INFRASTRUCTURE ONLY; numpy only; shares nothing with the HIP path.  Each function is the
definition written with numpy's own transpose / repeat / sum.

  * seq_a2a_pack_heads: what a GPU sends in the first SeqAlltoAll.  Its tokens hold all H heads,
    (s, H, d) token-major; message j holds head group j: (d_hp, H/d_hp, s, d).
  * seq_a2a_unpack_tokens: what it builds from the d_hp messages it receives, message i being
    GPU i's s tokens of this GPU's head group: (H/d_hp, d_hp * s, d), GPU i's tokens at
    positions i*s .. i*s+s-1.
  * the two inverses, used by the second SeqAlltoAll on the attention output and by the backward.
  * replicate_kv: (H_kv, s, d) -> (H_kv * rep, s, d), head h' = head h' // rep.
  * reduce_replicas: gradient of replicate_kv: the sum of the rep copies of every head (fp32,
    added in copy order).

Readings: the paper gives shapes only; which token goes where inside the re-partitioned
sequence (here: source GPU major) is this build's choice and is stated in the design notes.
"""
from __future__ import annotations

import numpy as np

__all__ = ["seq_a2a_pack_heads", "seq_a2a_unpack_tokens", "seq_a2a_pack_tokens", "seq_a2a_unpack_heads",
           "replicate_kv", "reduce_replicas"]


def seq_a2a_pack_heads(x: np.ndarray, d_hp: int) -> np.ndarray:
    s, H, d = x.shape
    return np.ascontiguousarray(x.reshape(s, d_hp, H // d_hp, d).transpose(1, 2, 0, 3))


def seq_a2a_unpack_tokens(msgs: np.ndarray) -> np.ndarray:
    d_hp, hl, s, d = msgs.shape
    return np.ascontiguousarray(msgs.transpose(1, 0, 2, 3)).reshape(hl, d_hp * s, d)


def seq_a2a_pack_tokens(x: np.ndarray, d_hp: int) -> np.ndarray:
    hl, S, d = x.shape
    return np.ascontiguousarray(x.reshape(hl, d_hp, S // d_hp, d).transpose(1, 0, 2, 3))


def seq_a2a_unpack_heads(msgs: np.ndarray) -> np.ndarray:
    d_hp, hl, s, d = msgs.shape
    return np.ascontiguousarray(msgs.transpose(2, 0, 1, 3)).reshape(s, d_hp * hl, d)


def replicate_kv(x: np.ndarray, rep: int) -> np.ndarray:
    return np.repeat(x, rep, axis=0)


def reduce_replicas(g: np.ndarray, rep: int) -> np.ndarray:
    hr, s, d = g.shape
    g = g.reshape(hr // rep, rep, s, d).astype(np.float32)
    acc = g[:, 0].copy()
    for r in range(1, rep):
        acc = acc + g[:, r]
    return acc
