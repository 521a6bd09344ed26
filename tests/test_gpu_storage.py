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


# --------------------------------------------------------------------------
# the weights as the forward kernels themselves see them
# --------------------------------------------------------------------------
def _weights_through_forward(mod, d_in, Gs, act, T):
    """Reads a module's weights through glowq_group_forward: X holds T rows of the
    identity (shifted call by call over the channels), r = 0, fp32 output, so that
    Y[t][o] is the one product 1.0 * w[o][c] plus exact zeros: the very value the
    kernel's own dequantiser fed to the matrix cores, unrounded by anything else."""
    from gpu_util import DeviceUnit, Workspace
    one = O.f64_to_bits(np.ones(1), act)[0]
    unit = dict(act=act, G=Gs, r=0, d_in=d_in, B=None, X=np.zeros((T, d_in), np.uint16),
                modules=[dict(mod, A=None)])
    du = DeviceUnit(unit)
    ws = Workspace([du.desc])
    d_out = mod["wq"].shape[0]
    seen = np.empty((d_out, d_in), np.float64)
    for c0 in range(0, d_in, T):
        n = min(T, d_in - c0)
        x = np.zeros((T, d_in), np.uint16)
        x[np.arange(n), c0 + np.arange(n)] = one
        du.X.copy_(torch.from_numpy(x.view(np.int16)).cuda())
        du.clear()
        G.glowq_group_forward(du.desc, False, ws.ptr, ws.bytes, stream())
        y = du.outputs()[0]
        seen[:, c0:c0 + n] = y[:n].T
    return seen


# token counts: 1-2, 3-4 (few-token streaming kernels), 16 and 32 (streaming kernel with
# one and two token blocks), 64 and d_in (tiled kernel with four and eight token blocks)
@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("Gs", [128, 64])
@pytest.mark.parametrize("T", [1, 2, 4, 16, 32, 64, 256])
def test_forward_kernels_multiply_with_the_stored_weight(act, Gs, T):
    """The dequantised weight is pinned bit for bit INSIDE every forward kernel (W4A16,
    Sec. 4.1).  Tiled kernels and every bfloat16 path form round_act((q - z) s) and must
    reproduce the oracle's bits; the binary16 streaming kernels (T <= 32) never round the
    weight: they multiply the exact integer (q - z) and apply s to the fp32 sum, so what
    they multiply with is (q - z) s itself, which fp32 holds exactly (5 + 11 bits)."""
    d_out, d_in = 48, 256
    rng = np.random.default_rng(3)
    q = rng.integers(0, 16, size=(d_out, d_in)).astype(np.uint8)
    # scales over the whole binary16 range that cannot overflow 15 s (subnormals included)
    s_bits = rng.integers(1, 0x6C00, size=(d_out, d_in // Gs)).astype(np.uint16)
    z = rng.integers(0, 16, size=(d_out, d_in // Gs)).astype(np.float64)
    z_bits = O.f64_to_bits(z, "f16")
    mod = dict(wq=O.pack_int4(q), scales=s_bits, zeros=z_bits)
    seen = _weights_through_forward(mod, d_in, Gs, act, T)
    unrounded = (q.astype(np.float64) - np.repeat(z, Gs, axis=1)) * \
        np.repeat(O.bits_to_f64(s_bits, "f16"), Gs, axis=1)
    if act == "f16" and T <= 32:
        ref = unrounded
        assert np.array_equal(ref, ref.astype(np.float32).astype(np.float64))   # exact in fp32
    else:
        ref = O.bits_to_f64(O.dequant_bits(q, s_bits, z_bits, Gs, act), act)
    bad = np.argwhere(seen != ref)
    assert bad.size == 0, (bad[:5], seen[tuple(bad[0])], ref[tuple(bad[0])])
