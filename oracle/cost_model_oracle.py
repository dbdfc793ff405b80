"""Plain oracle of the paper's performance model of 2D-Attention (Sec. "Performance Analysis":
"Computation Analysis", "P2P Communication Analysis", "SeqAlltoAll Communication Analysis").

TEST INFRASTRUCTURE ONLY: the product's calculator is the C function loong_cost_model; this
file restates the paper's formulas in the paper's notation, in Python floats, and shares
nothing with it.

Notation: sequence length S, hidden size D, H query heads, H_kv key/value heads,
d_sp = d_hp * d_cp, inner ring size w, alpha = forward seconds per unit of S^2 D.

Readings taken where the paper is silent (each is listed in the design notes):
  * transfer time of a message = latency + bytes / bandwidth;
  * the backward micro-step moves the K/V chunk and its gradient, twice the forward bytes
    (the gradients travel with the chunk, Sec. 3.1), and computes 3x as long;
  * T_SeqAlltoAll counts the forward and the backward phase: twice AlltoAll_Volume / bandwidth;
  * the replicated head count is max(H_kv, d_hp) (the smallest the paper allows).

Pins (tests/test_cost_model.py): the paper's worked size (GQA, 128K tokens, 8 GPUs: 64 MiB per
step), independence of Size(kv) from d_cp at fixed d_sp, GQA = MHA traffic at d_hp = H,
zero all-to-all traffic at d_hp = 1, compute-bound and communication-bound limits of
T_inner_ring, total compute d_cp * T_comp independent of w, and the whole objective with finite
links worked out by hand on two grids (communication-bound forward with compute-bound backward
inner ring and an all-to-all; a plain ring without one).
"""
from __future__ import annotations

__all__ = ["size_kv", "size_q", "alltoall_volume", "t_comp_fwd", "t_comp_bwd", "t_inner_ring", "objective"]


def size_kv(S, D, H, H_kv, d_hp, d_cp):
    """Bytes of one K/V chunk (two tensors, 16-bit elements): max(H_kv, d_hp) / H * 4 S D / d_sp."""
    return max(H_kv, d_hp) / H * 4.0 * S * D / (d_hp * d_cp)


def size_q(S, D, d_hp, d_cp):
    """Bytes of a Q chunk, equal to those of an output chunk: 2 S D / d_sp."""
    return 2.0 * S * D / (d_hp * d_cp)


def alltoall_volume(S, D, H, H_kv, d_hp, d_cp):
    """Bytes each GPU sends in one phase: sum over q, k, v, out of Size(i) * (d_hp - 1) / d_hp."""
    one_kv_tensor = size_kv(S, D, H, H_kv, d_hp, d_cp) / 2.0
    total = 2.0 * size_q(S, D, d_hp, d_cp) + 2.0 * one_kv_tensor
    return total * (d_hp - 1) / d_hp


def t_comp_fwd(alpha, S, D, d_hp, d_cp):
    """Forward time of one micro-step: alpha S^2 D / (d_cp d_sp)."""
    return alpha * S * S * D / (d_cp * d_hp * d_cp)


def t_comp_bwd(alpha, S, D, d_hp, d_cp):
    return 3.0 * t_comp_fwd(alpha, S, D, d_hp, d_cp)


def t_inner_ring(t_comp, t_p2p_inner, t_p2p_outer, w):
    """A (w - 1) + B with A = max(T_comp, T_P2P_inner), B = max(T_comp, T_P2P_outer)."""
    return max(t_comp, t_p2p_inner) * (w - 1) + max(t_comp, t_p2p_outer)


def objective(alpha, S, D, H, H_kv, d_hp, d_cp, w, bw_inner, bw_outer, bw_alltoall, latency=0.0):
    """T_SeqAlltoAll + (T_inner_ring^fwd + T_inner_ring^bwd) * d_cp / w, in seconds."""
    kv = size_kv(S, D, H, H_kv, d_hp, d_cp)
    fwd = t_inner_ring(t_comp_fwd(alpha, S, D, d_hp, d_cp), latency + kv / bw_inner, latency + kv / bw_outer, w)
    bwd = t_inner_ring(t_comp_bwd(alpha, S, D, d_hp, d_cp), latency + 2 * kv / bw_inner, latency + 2 * kv / bw_outer, w)
    t_a2a = 2.0 * alltoall_volume(S, D, H, H_kv, d_hp, d_cp) / bw_alltoall if d_hp > 1 else 0.0
    return t_a2a + (fwd + bwd) * d_cp / w
