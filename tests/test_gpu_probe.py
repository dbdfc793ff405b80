"""The matrix-only measurement aid (loong_mfma_probe) with operands of the caller's: what it leaves in
`sink` is fixed by the operand layout of v_mfma_f32_32x32x16_bf16 and can be worked out in integers."""
import numpy as np
import pytest
import torch

import paper_2406_18485_amd as P

pytestmark = pytest.mark.gpu


def test_probe_with_caller_operands_computes_the_product_of_its_two_operand_tiles():
    rng = np.random.default_rng(5)
    ints = rng.integers(-3, 4, size=(2, 64, 8))                     # [A | B][lane][element], exact in bf16
    operands = torch.tensor(ints.reshape(-1), dtype=torch.float32).bfloat16().cuda()
    assert operands.numel() * 2 == 2048
    wgs, iters = 3, 7
    sink = torch.zeros(wgs * 256, device="cuda:0")
    P.mfma_probe(wgs, iters, sink, operands)
    torch.cuda.synchronize()
    # lane l holds row (A) or column (B) l % 32 and the contraction indices 8 (l / 32) .. + 7
    A = np.zeros((32, 16), dtype=np.int64)
    B = np.zeros((16, 32), dtype=np.int64)
    for lane in range(64):
        A[lane % 32, 8 * (lane // 32):8 * (lane // 32) + 8] = ints[0, lane]
        B[8 * (lane // 32):8 * (lane // 32) + 8, lane % 32] = ints[1, lane]
    prod = A @ B * iters                                 # every chain repeats the product `iters` times
    # register v of a lane in half hh is row 8 (v / 4) + 4 hh + v % 4 of column lane % 32; the kernel adds up
    # registers 0, 5, 10, 15 of its four (identical) chains
    want = np.zeros(64, dtype=np.int64)
    for lane in range(64):
        hh, col = lane // 32, lane % 32
        want[lane] = sum(prod[8 * (v // 4) + 4 * hh + v % 4, col] for v in (0, 5, 10, 15))
    got = sink.cpu().numpy().reshape(wgs, 4, 64)
    assert np.array_equal(got, np.broadcast_to(want.astype(np.float32), got.shape))


def test_probe_with_built_in_operands_stays_finite():
    sink = torch.zeros(4 * 256, device="cuda:0")
    P.mfma_probe(4, 100, sink)
    torch.cuda.synchronize()
    assert torch.isfinite(sink).all() and (sink != 0).all()
