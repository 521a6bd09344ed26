"""GPU parity, storage format: the prepared layout unpacks to the oracle's q and
dequantises to the oracle's weight BIT FOR BIT (W4A16, Sec. 4.1)."""
import numpy as np
import pytest
import torch

import paper_2603_25385_amd as G
from oracle import glowq_oracle as O
from gpu_util import ACT_CODE, DeviceModule, stream

pytestmark = pytest.mark.gpu


def _module(seed, d_out, d_in, Gs, odd_scales=False):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((d_out, d_in)) * 0.02).astype(np.float32)
    q, s_bits, z_bits = O.quantize_rtn(W, Gs)
    if odd_scales:
        # scales across the whole binary16 range, subnormal included; every zero-point
        s_bits = rng.integers(1, 0x7BFF, size=s_bits.shape).astype(np.uint16)
        z_bits = O.f64_to_bits(rng.integers(0, 16, size=z_bits.shape).astype(np.float64), "f16")
        q = rng.integers(0, 16, size=q.shape).astype(np.uint8)
    return dict(wq=O.pack_int4(q), scales=s_bits, zeros=z_bits), q


@pytest.mark.parametrize("d_out,d_in,Gs", [(256, 256, 64), (40, 128, 128), (96, 1024, 128),
                                           (8, 128, 64), (1000, 384, 64)])
def test_unpack_bit_exact(d_out, d_in, Gs):
    mod, q = _module(1, d_out, d_in, Gs)
    dm = DeviceModule(mod, d_in, Gs)
    out = torch.empty((d_out, d_in), dtype=torch.uint8, device="cuda")
    G.glowq_debug_unpack(dm.prepared.data_ptr(), d_out, d_in, Gs, out.data_ptr(), stream())
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), q)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("d_out,d_in,Gs,odd", [(256, 256, 64, False), (40, 256, 128, False),
                                               (96, 1024, 128, True), (1000, 384, 64, True)])
def test_dequant_bit_exact(act, d_out, d_in, Gs, odd):
    mod, q = _module(2, d_out, d_in, Gs, odd)
    dm = DeviceModule(mod, d_in, Gs)
    out = torch.empty((d_out, d_in), dtype=torch.int16, device="cuda")
    G.glowq_debug_dequant(dm.prepared.data_ptr(), d_out, d_in, Gs, ACT_CODE[act], out.data_ptr(),
                          stream())
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    ref = O.dequant_bits(q, mod["scales"], mod["zeros"], Gs, act)
    # -0 and +0 are the same weight; compare values for zeros, bits elsewhere
    same = (got == ref) | (((got | ref) & 0x7FFF) == 0)
    assert same.all(), np.argwhere(~same)[:5]
