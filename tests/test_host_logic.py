"""CPU-only tests of the library's host side: exports, zigzag/ring order against the
oracle, descriptor validation and argument errors (none of these launches a kernel)."""
import os
import re

import numpy as np
import pytest

import oracle as orc
import paper_2406_18485_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "loong.h")).read()
    declared = set(re.findall(r"LOONG_API\s+[\w\s\*]+?\b(loong_\w+)\s*\(", hdr))
    assert declared == set(P.binding.EXPORTS)
    for name in declared:
        assert hasattr(P.binding.lib, name), name
    assert P.version() >= 100


@pytest.mark.parametrize("cp,w", [(1, 1), (2, 1), (4, 4), (4, 2), (8, 4), (8, 8), (16, 4), (6, 3), (32, 32), (12, 2)])
def test_zigzag_mask_matches_oracle(cp, w):
    for r in range(cp):
        order = orc.double_ring_sources(cp, w, r)
        for t in range(cp):
            z = P.zigzag_mask(cp, w, r, t)
            assert z["src_rank"] == order[t]
            assert z["q_chunk"] == orc.zigzag_chunk_ids(cp, r)
            assert z["kv_chunk"] == orc.zigzag_chunk_ids(cp, order[t])
            cls = orc.quadrant_classes(z["q_chunk"], z["kv_chunk"])
            assert tuple(int(x) for x in cls.reshape(-1)) == z["block_class"]
            assert (P.SKIP, P.FULL, P.DIAG) == (orc.SKIP, orc.FULL, orc.DIAG)


def test_zigzag_mask_first_benchmark_case_and_null_outputs():
    z = P.zigzag_mask(4, 4, 0, 0)
    assert z["q_chunk"] == (0, 7) and z["src_rank"] == 0 and z["block_class"] == (P.DIAG, P.SKIP, P.FULL, P.DIAG)
    assert [P.zigzag_mask(4, 4, 0, t)["src_rank"] for t in range(4)] == [0, 3, 2, 1]
    assert P.binding.lib.loong_zigzag_mask(4, 2, 1, 3, None, None, None, None) == P.OK


@pytest.mark.parametrize("args", [(0, 1, 0, 0), (4, 3, 0, 0), (4, 0, 0, 0), (4, 2, 4, 0), (4, 2, -1, 0), (4, 2, 0, 4), (4, 2, 0, -1)])
def test_zigzag_mask_rejects_bad_arguments(args):
    with pytest.raises(P.LoongError) as e:
        P.zigzag_mask(*args)
    assert e.value.code == P.E_SHAPE and P.last_error()


def _good(**kw):
    base = dict(batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, q_len=512, kv_len=512, dtype=P.BF16,
                softmax_scale=0.1, causal=True, chunk_len=256, q_chunk=(1, 6), kv_chunk=(0, 7))
    base.update(kw)
    return P.make_desc(**base)


def test_validate_accepts_the_benchmark_shapes():
    assert P.validate_step(_good()) == P.OK
    assert P.validate_step(_good(dtype=P.FP32, head_dim=64, n_q_heads=2, n_kv_heads=2, q_len=256, kv_len=256, chunk_len=128)) == P.OK
    assert P.validate_step(_good(dtype=P.FP16)) == P.OK and P.validate_step(_good(dtype=P.FP16, head_dim=64)) == P.OK
    assert P.validate_step(_good(causal=False, q_len=77, kv_len=0, chunk_len=0)) == P.OK
    assert P.validate_step(_good(batch=0)) == P.OK


@pytest.mark.parametrize("kw,code", [
    (dict(dtype=7), P.E_DTYPE),
    (dict(dtype=3), P.E_DTYPE),
    (dict(dtype=P.FP16, head_dim=96), P.E_UNSUPPORTED),
    (dict(head_dim=96), P.E_UNSUPPORTED),
    (dict(dtype=P.FP32, head_dim=130), P.E_UNSUPPORTED),
    (dict(dtype=P.FP32, head_dim=256), P.E_UNSUPPORTED),
    (dict(n_q_heads=7), P.E_UNSUPPORTED),
    (dict(n_kv_heads=0), P.E_SHAPE),
    (dict(q_len=-1), P.E_SHAPE),
    (dict(q_len=511), P.E_SHAPE),
    (dict(kv_len=510), P.E_SHAPE),
    (dict(q_chunk=(1, 1)), P.E_SHAPE),
    (dict(kv_chunk=(-1, 7)), P.E_SHAPE),
    (dict(softmax_scale=0.0), P.E_SHAPE),
    (dict(softmax_scale=float("nan")), P.E_SHAPE),
    (dict(q_stride=(8 * 512 * 128, 512 * 128, 100)), P.E_ALIGN),
    (dict(kv_stride=(2 * 512 * 128, 512 * 128 + 4, 128)), P.E_ALIGN),
    (dict(o_stride=(8 * 512 * 128, 512 * 128, 64)), P.E_SHAPE),
    (dict(causal=False, q_len=(1 << 24) + 1, chunk_len=0), P.E_UNSUPPORTED),
])
def test_validate_rejects(kw, code):
    assert P.validate_step(_good(**kw)) == code
    assert P.last_error()


def test_entry_points_fail_before_any_launch_on_bad_arguments():
    lib = P.binding.lib
    d = _good()
    import ctypes as C
    # NULL tensors
    assert lib.loong_attn_step_fwd(C.byref(d), None, None, None, None, None, None) == P.E_NULL
    assert lib.loong_attn_step_bwd(C.byref(d), *([None] * 11), 0, None) == P.E_NULL
    assert lib.loong_bwd_delta(C.byref(d), None, None, None, None) == P.E_NULL
    assert lib.loong_lse_merge(4, 128, None, None, None, None, None) == P.E_NULL
    assert lib.loong_init_running(4, 128, None, None, None) == P.E_NULL
    assert lib.loong_finalize_out(4, 128, None, None, P.BF16, None) == P.E_NULL
    assert lib.loong_attn_step_fwd(None, 16, 16, 16, 16, 16, None) == P.E_NULL
    # misaligned pointers, bad sizes: fake non-NULL addresses are never dereferenced on these paths
    assert lib.loong_attn_step_fwd(C.byref(d), 0x1008, 0x1000, 0x1000, 0x1000, 0x1000, None) == P.E_ALIGN
    assert lib.loong_lse_merge(4, 130, 0x1000, 0x1000, 0x1000, 0x1000, None) == P.E_UNSUPPORTED
    assert lib.loong_lse_merge(-1, 128, 0x1000, 0x1000, 0x1000, 0x1000, None) == P.E_SHAPE
    assert lib.loong_lse_merge(4, 128, 0x1004, 0x1000, 0x1000, 0x1000, None) == P.E_ALIGN
    assert lib.loong_finalize_out(4, 128, 0x1000, 0x1000, 9, None) == P.E_DTYPE
    assert lib.loong_finalize_out(4, 100, 0x1000, 0x1000, P.BF16, None) == P.E_UNSUPPORTED
    # zero-sized work returns OK without touching the (fake) pointers
    assert lib.loong_lse_merge(0, 128, 0x1000, 0x1000, 0x1000, 0x1000, None) == P.OK
    assert lib.loong_attn_step_fwd(C.byref(_good(batch=0)), 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, None) == P.OK
    dd = _good(flags=P.COMPUTE_DELTA)
    assert lib.loong_attn_step_bwd(C.byref(dd), 16, 16, 16, None, 16, 16, 16, 16, 16, 16, None, 0, None) == P.E_NULL
    # the one-sided backward flags: exclusive, and each lifts the NULL check of the other side's outputs only
    both = _good(flags=P.BWD_ONLY_DKV | P.BWD_ONLY_DQ)
    assert lib.loong_attn_step_bwd(C.byref(both), *([0x1000] * 10), None, 0, None) == P.E_UNSUPPORTED
    z = _good(batch=0, flags=P.BWD_ONLY_DKV)
    assert lib.loong_attn_step_bwd(C.byref(z), 0x1000, 0x1000, 0x1000, None, 0x1000, 0x1000, 0x1000, None, 0x1000, 0x1000, None, 0, None) == P.OK
    assert lib.loong_attn_step_bwd(C.byref(z), 0x1000, 0x1000, 0x1000, None, 0x1000, 0x1000, 0x1000, None, None, 0x1000, None, 0, None) == P.E_NULL
    z = _good(batch=0, flags=P.BWD_ONLY_DQ)
    assert lib.loong_attn_step_bwd(C.byref(z), 0x1000, 0x1000, 0x1000, None, 0x1000, 0x1000, 0x1000, 0x1000, None, None, None, 0, None) == P.OK
    assert lib.loong_attn_step_bwd(C.byref(z), 0x1000, 0x1000, 0x1000, None, 0x1000, 0x1000, 0x1000, None, None, None, None, 0, None) == P.E_NULL


def test_error_text_is_per_call():
    assert P.validate_step(_good(head_dim=96)) != P.OK and "head_dim" in P.last_error()
    assert P.validate_step(_good()) == P.OK and P.last_error() == ""


def test_layout_and_probe_entry_points_validate_before_touching_a_device():
    import ctypes as C
    lib = P.binding.lib
    a3 = C.c_int64 * 3
    ok = a3(16, 16, 16)
    assert lib.loong_permute_rows(a3(1, 1, 1), ok, ok, 16, None, 0x1000, None) == P.E_NULL
    assert lib.loong_permute_rows(a3(1, 1, 1), ok, a3(16, 16, 8), 16, 0x1000, 0x2000, None) == P.E_ALIGN
    assert lib.loong_permute_rows(a3(1, 1, 1), ok, ok, 24, 0x1000, 0x2000, None) == P.E_ALIGN
    assert lib.loong_permute_rows(a3(-1, 1, 1), ok, ok, 16, 0x1000, 0x2000, None) == P.E_SHAPE
    assert lib.loong_permute_rows(a3(0, 1, 1), ok, ok, 16, 0x1000, 0x2000, None) == P.OK
    assert lib.loong_reduce_replicas(2, 0, 4, 0x1000, 0x2000, None) == P.E_SHAPE
    assert lib.loong_reduce_replicas(2, 2, 6, 0x1000, 0x2000, None) == P.E_ALIGN
    assert lib.loong_reduce_replicas(0, 2, 4, 0x1000, 0x2000, None) == P.OK
    assert lib.loong_mfma_probe(0, 1, None, 0x1000, None) == P.E_SHAPE
    assert lib.loong_mfma_probe(1, 1, None, None, None) == P.E_NULL
    assert lib.loong_mfma_probe(1, 1, 0x1008, 0x1000, None) == P.E_ALIGN


def test_workspace_bytes_follows_the_split_of_the_query_loops():
    """Few key tiles (fewer than CUs): the query loops are shared and partial sums are parked; many: nothing is."""
    per_item = 8 * (128 // 32) * 16 * 64 * 4            # one (key tile, split) slot: eight waves' accumulators
    counters = 16384 * 4                                 # the arrival counters in front of the partial sums
    small = _good(n_q_heads=8, n_kv_heads=8, q_len=4096, kv_len=4096, chunk_len=2048, causal=1,
                  q_chunk=(7, 8), kv_chunk=(3, 12))      # both local chunks see the early key chunk only: 16 tiles x 8 heads
    assert P.workspace_bytes(small) == counters + 128 * 2 * per_item
    big = _good(n_q_heads=8, n_kv_heads=8, q_len=16384, kv_len=16384, chunk_len=8192, causal=1,
                q_chunk=(0, 31), kv_chunk=(5, 26))
    assert P.workspace_bytes(big) == 0
    big.flags = P.BWD_ONLY_DQ
    small.flags = P.BWD_ONLY_DQ
    assert P.workspace_bytes(small) == 0
    assert P.workspace_bytes(_good(dtype=P.FP32, head_dim=64, n_q_heads=2, n_kv_heads=2, q_len=256, kv_len=256, chunk_len=128)) == 0
    lib = P.binding.lib
    import ctypes as C
    assert lib.loong_workspace_bytes(C.byref(small), None) == P.E_NULL


def test_backward_step_rejects_a_missing_or_small_workspace_before_any_launch():
    """The step that shares query loops needs caller-owned scratch: without it, or with too little or a misaligned
    block, the call returns an argument error and enqueues nothing (fake addresses are never dereferenced)."""
    import ctypes as C
    lib = P.binding.lib
    small = _good(n_q_heads=8, n_kv_heads=8, q_len=4096, kv_len=4096, chunk_len=2048, causal=1,
                  q_chunk=(7, 8), kv_chunk=(3, 12))
    need = P.workspace_bytes(small)
    assert need > 0
    ptrs = [0x1000] * 3 + [None] + [0x1000] * 6
    assert lib.loong_attn_step_bwd(C.byref(small), *ptrs, None, 0, None) == P.E_NULL and "workspace" in P.last_error()
    assert lib.loong_attn_step_bwd(C.byref(small), *ptrs, 0x1000, need - 1, None) == P.E_SHAPE and str(need) in P.last_error()
    assert lib.loong_attn_step_bwd(C.byref(small), *ptrs, 0x1008, need, None) == P.E_ALIGN
    assert lib.loong_attn_step_bwd(C.byref(small), *ptrs, 0x1000, -1, None) == P.E_SHAPE
    # the dQ half alone needs none
    small.flags = P.BWD_ONLY_DQ
    assert P.workspace_bytes(small) == 0


def test_key_split_override_is_validated():
    assert P.validate_step(_good(flags=P.key_splits(1))) == P.OK
    assert P.validate_step(_good(flags=P.key_splits(2) | P.FUSE_MERGE)) == P.OK
    assert P.validate_step(_good(flags=P.key_splits(4))) == P.OK
    for bad in (3, 5, 6, 7):
        assert P.validate_step(_good(flags=P.key_splits(bad))) == P.E_UNSUPPORTED and "LOONG_KEY_SPLITS" in P.last_error()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)


def test_package_fails_loudly_without_the_library(tmp_path):
    """A copy of the package without libloong.so: the build module imports, anything else raises ImportError."""
    import shutil
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = tmp_path / "paper_2406_18485_amd"
    shutil.copytree(os.path.join(root, "paper_2406_18485_amd"), pkg,
                    ignore=shutil.ignore_patterns("*.so", "_build", "__pycache__"))
    code = ("import paper_2406_18485_amd as P\n"
            "import paper_2406_18485_amd.build\n"
            "try:\n    P.version()\n    print('NO ERROR')\nexcept ImportError as e:\n    print('ImportError', 'no fallback' in str(e))\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=tmp_path, capture_output=True, text=True, timeout=120)
    assert r.stdout.strip() == "ImportError True", r.stdout + r.stderr
