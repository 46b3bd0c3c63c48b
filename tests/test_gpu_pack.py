"""Stage-boundary packing of (C, F) on the GPU against oracle/pack.py: the packed bytes are compared bit for bit,
unpacking an oracle-made buffer gives the oracle's arrays, and the round trip is the identity."""
import numpy as np
import pytest
import torch

from oracle import pack as opack
from paper_2012_13846_amd import spgen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    from paper_2012_13846_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("n,c,bf16", [(0, 8, False), (1, 1, True), (1001, 5, False), (777, 3, True), (100848, 64, False),
                                      (373607, 64, True), (4099, 256, True)])
def test_pack_unpack_match_oracle(sp, n, c, bf16):
    rng = np.random.default_rng(n + c)
    coords = rng.integers(-30000, 30000, (n, 4)).astype(np.int32)
    coords[:, 0] = rng.integers(0, 8, n)
    feats = spgen.features(n + 7, n, c, bf16)
    bits = spgen.f32_to_bf16_bits(feats) if bf16 else feats
    dtype = 1 if bf16 else 0
    want = opack.pack(coords, bits, dtype, 2)
    d_coords = torch.from_numpy(coords).cuda()
    d_feats = torch.from_numpy(feats).cuda().to(torch.bfloat16 if bf16 else torch.float32)
    buf = sp.sp_pack(d_coords, d_feats, 2)
    assert buf.numel() == len(want) == opack.packed_bytes(n, c, dtype)
    assert np.array_equal(buf.cpu().numpy(), want)
    # unpack a buffer the oracle made
    c2, f2, ts2 = sp.sp_unpack(torch.from_numpy(want).cuda())
    assert ts2 == 2 and np.array_equal(c2.cpu().numpy(), coords)
    got_bits = f2.view(torch.int16).cpu().numpy().view(np.uint16) if bf16 else f2.cpu().numpy()
    assert np.array_equal(got_bits, bits)
    # round trip on the device
    c3, f3, ts3 = sp.sp_unpack(buf)
    assert torch.equal(c3, d_coords) and torch.equal(f3, d_feats) and ts3 == 2


def test_unaligned_feature_pointer_and_bad_buffers(sp):
    n, c = 300, 3
    coords = torch.zeros((n, 4), dtype=torch.int32, device="cuda")
    backing = torch.arange(n * c + 1, dtype=torch.float32, device="cuda")
    feats = backing[1:].view(n, c)                    # 4-byte aligned only
    buf = sp.sp_pack(coords, feats, 1)
    want = opack.pack(coords.cpu().numpy(), feats.cpu().numpy(), 0, 1)
    assert np.array_equal(buf.cpu().numpy(), want)
    bad = buf.clone()
    bad[0] = 0
    with pytest.raises(sp.SpError) as e:
        sp.sp_unpack(bad)
    assert e.value.code == -1
