"""SeqAlltoAll local re-arrangements, KV replication and its gradient reduction: HIP path against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

import paper_2406_18485_amd as P
from oracle import layout_oracle as lo

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


@pytest.mark.parametrize("s,H,d,d_hp,esize", [(257, 8, 128, 4, 2), (64, 32, 128, 8, 2), (33, 4, 64, 1, 2), (100, 6, 32, 3, 4)])
def test_first_and_second_all_to_all_layouts(s, H, d, d_hp, esize):
    rng = np.random.default_rng(s + H)
    np_t = np.uint16 if esize == 2 else np.float32
    x = rng.integers(0, 60000, (s, H, d)).astype(np_t) if esize == 2 else rng.standard_normal((s, H, d)).astype(np_t)
    hl, e = H // d_hp, esize
    # heads of (s, H, d) into d_hp messages (d_hp, hl, s, d)
    msgs = torch.zeros(d_hp, hl, s, d, dtype=torch.from_numpy(x).dtype, device=DEV)
    P.permute_rows((d_hp, hl, s), (hl * d * e, d * e, H * d * e), (hl * s * d * e, s * d * e, d * e), d * e, _dev(x), msgs)
    torch.cuda.synchronize()
    want = lo.seq_a2a_pack_heads(x, d_hp)
    assert np.array_equal(msgs.cpu().numpy(), want)
    # d_hp received messages into (hl, d_hp*s, d)
    loc = torch.zeros(hl, d_hp * s, d, dtype=msgs.dtype, device=DEV)
    P.permute_rows((d_hp, hl, s), (hl * s * d * e, s * d * e, d * e), (s * d * e, d_hp * s * d * e, d * e), d * e, msgs, loc)
    torch.cuda.synchronize()
    want_loc = lo.seq_a2a_unpack_tokens(want)
    assert np.array_equal(loc.cpu().numpy(), want_loc)
    # the way back: token groups into messages, messages into token-major
    back = torch.zeros(d_hp, hl, s, d, dtype=msgs.dtype, device=DEV)
    P.permute_rows((d_hp, hl, s), (s * d * e, d_hp * s * d * e, d * e), (hl * s * d * e, s * d * e, d * e), d * e, loc, back)
    out = torch.zeros(s, H, d, dtype=msgs.dtype, device=DEV)
    P.permute_rows((d_hp, hl, s), (hl * s * d * e, s * d * e, d * e), (hl * d * e, d * e, H * d * e), d * e, back, out)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy(), lo.seq_a2a_pack_tokens(want_loc, d_hp))
    assert np.array_equal(out.cpu().numpy(), lo.seq_a2a_unpack_heads(back.cpu().numpy())) and np.array_equal(out.cpu().numpy(), x)


@pytest.mark.parametrize("hkv,rep,s,d", [(2, 4, 130, 128), (8, 1, 17, 64), (1, 8, 1000, 128)])
def test_kv_replication_and_gradient_reduction(hkv, rep, s, d):
    rng = np.random.default_rng(hkv * 10 + rep)
    x = rng.integers(0, 60000, (hkv, s, d)).astype(np.uint16)
    out = torch.zeros(hkv * rep, s, d, dtype=torch.uint16, device=DEV)
    P.permute_rows((hkv, rep, s), (s * d * 2, 0, d * 2), (rep * s * d * 2, s * d * 2, d * 2), d * 2, _dev(x), out)
    g = rng.standard_normal((hkv * rep, s, d)).astype(np.float32)
    red = torch.full((hkv, s, d), 7.0, device=DEV)
    P.reduce_replicas(hkv, rep, s * d, _dev(g), red)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), lo.replicate_kv(x, rep))
    assert np.array_equal(red.cpu().numpy(), lo.reduce_replicas(g, rep))   # same order of fp32 additions


def test_empty_and_error_paths():
    z = torch.zeros(16, device=DEV)
    P.permute_rows((0, 3, 4), (16, 16, 16), (16, 16, 16), 16, z, z)          # nothing to do
    P.reduce_replicas(0, 2, 4, z, z)
    with pytest.raises(P.LoongError):
        P.permute_rows((1, 1, 1), (16, 16, 16), (16, 16, 8), 16, z, z)       # stride not a multiple of 16
    with pytest.raises(P.LoongError):
        P.permute_rows((1, 1, 1), (16, 16, 16), (16, 16, 16), 24, z, z)      # row not a multiple of 16
    with pytest.raises(P.LoongError):
        P.reduce_replicas(2, 0, 4, z, z)
    with pytest.raises(P.LoongError):
        P.reduce_replicas(2, 2, 6, z, z)
