"""ctypes binding of libloong.so: same names as the C ABI, argument marshalling only.

Every step of the path runs inside the library's HIP kernels; this module converts
Python/torch arguments to pointers and sizes and raises on a non-zero status.  There is
no CPU fallback: if the library is missing, importing this module fails.
"""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libloong.so")

OK, E_NULL, E_SHAPE, E_UNSUPPORTED, E_ALIGN, E_DTYPE, E_HIP = 0, -1, -2, -3, -4, -5, -6
BF16, FP32, FP16 = 0, 1, 2
SKIP, FULL, DIAG = 0, 1, 2
FUSE_MERGE, ACCUM_DKV, COMPUTE_DELTA, BWD_ONLY_DKV, BWD_ONLY_DQ = 1, 2, 4, 8, 16
KEY_SPLITS_SHIFT = 8


def key_splits(n: int) -> int:
    """LOONG_KEY_SPLITS(n): flag bits that force n (1, 2 or 4) key splits in the forward and dQ kernels."""
    return n << KEY_SPLITS_SHIFT


EXPORTS = (
    "loong_zigzag_mask", "loong_attn_step_fwd", "loong_lse_merge", "loong_attn_step_bwd",
    "loong_bwd_delta", "loong_init_running", "loong_finalize_out", "loong_validate_step",
    "loong_last_error", "loong_version", "loong_mfma_probe", "loong_cost_model", "loong_cost_search",
    "loong_permute_rows", "loong_reduce_replicas", "loong_workspace_bytes", "loong_attn_step_bwd_static",
)


class LoongError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libloong status {code}: {text}")
        self.code = code


class StepDesc(C.Structure):
    """Mirror of loong_step_desc."""
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("q_len", C.c_int32), ("kv_len", C.c_int32), ("chunk_len", C.c_int32),
        ("q_chunk", C.c_int32 * 2), ("kv_chunk", C.c_int32 * 2),
        ("causal", C.c_int32), ("dtype", C.c_int32), ("softmax_scale", C.c_float), ("flags", C.c_int32),
        ("q_stride", C.c_int64 * 3), ("kv_stride", C.c_int64 * 3), ("o_stride", C.c_int64 * 3),
    ]


class CostIn(C.Structure):
    """Mirror of loong_cost_in."""
    _fields_ = [("S", C.c_double), ("D", C.c_double), ("H", C.c_int32), ("H_kv", C.c_int32), ("d_hp", C.c_int32),
                ("d_cp", C.c_int32), ("w", C.c_int32), ("alpha_fwd", C.c_double), ("bw_p2p_inner", C.c_double),
                ("bw_p2p_outer", C.c_double), ("bw_alltoall", C.c_double), ("latency", C.c_double)]


class CostOut(C.Structure):
    """Mirror of loong_cost_out."""
    _fields_ = [(n, C.c_double) for n in (
        "size_kv", "size_q", "alltoall_volume", "t_comp_fwd", "t_comp_bwd", "t_p2p_inner_fwd", "t_p2p_outer_fwd",
        "t_p2p_inner_bwd", "t_p2p_outer_bwd", "t_inner_ring_fwd", "t_inner_ring_bwd", "t_seq_alltoall", "objective")]


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2406_18485_amd.build` "
        "(there is no fallback implementation)")

# One HIP runtime per process: torch ships its own copy and the library must bind to the same one
# (loaded the other way round, the library pulls in the system's copy first, torch then runs on a
# runtime it was not built for, and the library's device queries fail).  So torch goes first
# wherever it is installed; without torch the system's runtime is the only one.
try:
    import torch  # noqa: F401
except ImportError:
    pass

lib = C.CDLL(LIB_PATH)

_vp, _i32, _i64 = C.c_void_p, C.c_int32, C.c_int64
lib.loong_zigzag_mask.argtypes = [_i32, _i32, _i32, _i32, C.POINTER(_i32), C.POINTER(_i32), C.POINTER(_i32),
                                  C.POINTER(C.c_uint8)]
lib.loong_attn_step_fwd.argtypes = [C.POINTER(StepDesc), _vp, _vp, _vp, _vp, _vp, _vp]
lib.loong_lse_merge.argtypes = [_i64, _i32, _vp, _vp, _vp, _vp, _vp]
lib.loong_attn_step_bwd.argtypes = [C.POINTER(StepDesc)] + [_vp] * 11 + [_i64, _vp]
lib.loong_attn_step_bwd_static.argtypes = [C.POINTER(StepDesc)] + [_vp] * 11
lib.loong_bwd_delta.argtypes = [C.POINTER(StepDesc), _vp, _vp, _vp, _vp]
lib.loong_init_running.argtypes = [_i64, _i32, _vp, _vp, _vp]
lib.loong_finalize_out.argtypes = [_i64, _i32, _vp, _vp, _i32, _vp]
lib.loong_validate_step.argtypes = [C.POINTER(StepDesc)]
lib.loong_mfma_probe.argtypes = [_i32, _i32, _vp, _vp, _vp]
lib.loong_workspace_bytes.argtypes = [C.POINTER(StepDesc), C.POINTER(C.c_int64)]
lib.loong_permute_rows.argtypes = [C.POINTER(_i64), C.POINTER(_i64), C.POINTER(_i64), _i64, _vp, _vp, _vp]
lib.loong_reduce_replicas.argtypes = [_i64, _i32, _i64, _vp, _vp, _vp]
lib.loong_cost_model.argtypes = [C.POINTER(CostIn), C.POINTER(CostOut)]
lib.loong_cost_search.argtypes = [C.POINTER(CostIn), _i32, _i32, C.POINTER(CostIn), C.POINTER(CostOut)]
lib.loong_last_error.restype = C.c_char_p
for _n in EXPORTS:
    if _n != "loong_last_error":
        getattr(lib, _n).restype = C.c_int


def _ptr(x):
    """Device pointer of a torch tensor, or an int / None passed through."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc: int):
    if rc != 0:
        raise LoongError(rc, lib.loong_last_error().decode())


def last_error() -> str:
    return lib.loong_last_error().decode()


def version() -> int:
    return lib.loong_version()


def _cost_in(S, D, H, H_kv, alpha_fwd, bw_p2p_inner, bw_p2p_outer, bw_alltoall, latency=0.0, d_hp=1, d_cp=1, w=1):
    return CostIn(S=S, D=D, H=H, H_kv=H_kv, d_hp=d_hp, d_cp=d_cp, w=w, alpha_fwd=alpha_fwd, bw_p2p_inner=bw_p2p_inner,
                  bw_p2p_outer=bw_p2p_outer, bw_alltoall=bw_alltoall, latency=latency)


def _as_dict(st) -> dict:
    return {n: getattr(st, n) for n, _ in st._fields_}


def cost_model(**kw) -> dict:
    """loong_cost_model: keyword arguments are the fields of loong_cost_in; returns loong_cost_out as a dict."""
    out = CostOut()
    _check(lib.loong_cost_model(C.byref(_cost_in(**kw)), C.byref(out)))
    return _as_dict(out)


def cost_search(d_sp: int, max_w: int, **kw) -> dict:
    """loong_cost_search: the best grid for d_sp GPUs; returns the outputs plus d_hp, d_cp, w."""
    best_in, best_out = CostIn(), CostOut()
    _check(lib.loong_cost_search(C.byref(_cost_in(**kw)), d_sp, max_w, C.byref(best_in), C.byref(best_out)))
    res = _as_dict(best_out)
    res.update(d_hp=best_in.d_hp, d_cp=best_in.d_cp, w=best_in.w)
    return res


def permute_rows(n, in_stride, out_stride, row_bytes: int, src, dst, stream=None):
    """loong_permute_rows: n, in_stride, out_stride are 3-sequences (strides in bytes)."""
    a3 = _i64 * 3
    _check(lib.loong_permute_rows(a3(*n), a3(*in_stride), a3(*out_stride), row_bytes, _ptr(src), _ptr(dst), _stream(stream)))


def reduce_replicas(heads: int, rep: int, elems_per_head: int, src, dst, stream=None):
    _check(lib.loong_reduce_replicas(heads, rep, elems_per_head, _ptr(src), _ptr(dst), _stream(stream)))


def workspace_bytes(desc) -> int:
    """Bytes of caller-owned workspace the backward step of this descriptor needs (0: none)."""
    n = C.c_int64(0)
    _check(lib.loong_workspace_bytes(C.byref(desc), C.byref(n)))
    return n.value


def mfma_probe(workgroups: int, iters: int, sink, operands=None, stream=None):
    """`operands`: None (built-in, nearly constant) or a device tensor of 2048 bytes (see loong_mfma_probe)."""
    _check(lib.loong_mfma_probe(workgroups, iters, _ptr(operands), _ptr(sink), _stream(stream)))


def make_desc(*, batch, n_q_heads, n_kv_heads, head_dim, q_len, kv_len, dtype, softmax_scale,
              causal=False, chunk_len=0, q_chunk=(0, 0), kv_chunk=(0, 0), flags=0,
              q_stride=None, kv_stride=None, o_stride=None) -> StepDesc:
    """Descriptor with contiguous [batch, head, token, head_dim] strides unless given."""
    def contig(h, n):
        return (h * n * head_dim, n * head_dim, head_dim)
    d = StepDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = batch, n_q_heads, n_kv_heads, head_dim
    d.q_len, d.kv_len, d.chunk_len = q_len, kv_len, chunk_len
    d.q_chunk[:] = q_chunk
    d.kv_chunk[:] = kv_chunk
    d.causal, d.dtype, d.softmax_scale, d.flags = int(causal), dtype, softmax_scale, flags
    d.q_stride[:] = q_stride or contig(n_q_heads, q_len)
    d.kv_stride[:] = kv_stride or contig(n_kv_heads, kv_len)
    d.o_stride[:] = o_stride or contig(n_q_heads, q_len)
    return d


def validate_step(desc: StepDesc) -> int:
    """Status of the descriptor check (no exception: callers test error codes)."""
    return lib.loong_validate_step(C.byref(desc))


def zigzag_mask(cp: int, inner_w: int, rank: int, step: int) -> dict:
    src = _i32()
    qc = (_i32 * 2)()
    kc = (_i32 * 2)()
    cls = (C.c_uint8 * 4)()
    _check(lib.loong_zigzag_mask(cp, inner_w, rank, step, C.byref(src), qc, kc, cls))
    return {"src_rank": src.value, "q_chunk": (qc[0], qc[1]), "kv_chunk": (kc[0], kc[1]),
            "block_class": tuple(cls)}


def attn_step_fwd(desc: StepDesc, q, k, v, out, lse, stream=None):
    _check(lib.loong_attn_step_fwd(C.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _stream(stream)))


def lse_merge(rows: int, head_dim: int, out, lse, block_out, block_lse, stream=None):
    _check(lib.loong_lse_merge(rows, head_dim, _ptr(out), _ptr(lse), _ptr(block_out), _ptr(block_lse),
                               _stream(stream)))


def attn_step_bwd(desc: StepDesc, q, k, v, o, d_o, lse, delta, dq, dk, dv, workspace=None, workspace_bytes=None,
                  stream=None):
    """`workspace`: a device tensor (its size in bytes is taken from it) or a raw pointer with `workspace_bytes`."""
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None or isinstance(workspace, int) else workspace.numel() * workspace.element_size()
    _check(lib.loong_attn_step_bwd(C.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse),
                                   _ptr(delta), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace), workspace_bytes,
                                   _stream(stream)))


STATIC_SCRATCH_BYTES = (64 << 20) + 65536


def attn_step_bwd_static(desc: StepDesc, q, k, v, o, d_o, lse, delta, dq, dk, dv, stream=None):
    """loong_attn_step_bwd_static: the backward step on the library's static scratch array (no workspace)."""
    _check(lib.loong_attn_step_bwd_static(C.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse),
                                          _ptr(delta), _ptr(dq), _ptr(dk), _ptr(dv), _stream(stream)))


def bwd_delta(desc: StepDesc, o, d_o, delta, stream=None):
    _check(lib.loong_bwd_delta(C.byref(desc), _ptr(o), _ptr(d_o), _ptr(delta), _stream(stream)))


def init_running(rows: int, head_dim: int, out, lse, stream=None):
    _check(lib.loong_init_running(rows, head_dim, _ptr(out), _ptr(lse), _stream(stream)))


def finalize_out(rows: int, head_dim: int, out, o, dtype: int, stream=None):
    _check(lib.loong_finalize_out(rows, head_dim, _ptr(out), _ptr(o), dtype, _stream(stream)))
