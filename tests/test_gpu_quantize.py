"""GPU parity of the round-to-nearest INT4 quantiser (Sec. 4.1) with the oracle's: codes,
scales and zero-points bit for bit, on ordinary weights and on the groups where a rounding
decision is closest (ties, a zero range, one-sided ranges, the scale floor, a scale past the
binary16 range)."""
import numpy as np
import pytest
import torch

import paper_2603_25385_amd as G
from oracle import glowq_oracle as O
from gpu_util import stream

pytestmark = pytest.mark.gpu


def gpu_quantize(W, Gs):
    d_out, d_in = W.shape
    w = torch.from_numpy(np.ascontiguousarray(W, np.float32)).cuda()
    wq = torch.full((d_out + 1, d_in // 8), -1, dtype=torch.int32, device="cuda")
    sc = torch.full((d_out + 1, d_in // Gs), -1, dtype=torch.int16, device="cuda")
    zp = torch.full((d_out + 1, d_in // Gs), -1, dtype=torch.int16, device="cuda")
    G.glowq_quantize_rtn(w.data_ptr(), d_out, d_in, Gs, wq.data_ptr(), sc.data_ptr(), zp.data_ptr(), stream())
    torch.cuda.synchronize()
    assert (wq[-1] == -1).all() and (sc[-1] == -1).all() and (zp[-1] == -1).all()
    return (wq[:-1].cpu().numpy().view(np.uint32), sc[:-1].cpu().numpy().view(np.uint16),
            zp[:-1].cpu().numpy().view(np.uint16))


def crafted(d_out, d_in, Gs, seed):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((d_out, d_in)) * 0.02).astype(np.float32)
    g = lambda i: slice(i * Gs, (i + 1) * Gs)
    W[0, g(0)] = 0.0                                              # zero range: the scale floor
    W[1, g(0)] = np.abs(W[1, g(0)])                               # one-sided, positive
    W[2, g(0)] = -np.abs(W[2, g(0)])                              # one-sided, negative
    W[3, g(1)] = rng.standard_normal(Gs) * 2e6                    # scale past the binary16 range
    W[4, g(1)] = rng.standard_normal(Gs) * 1e-7                   # below the floor of the scale
    k = rng.integers(0, 15, Gs)
    W[5, g(0)] = (k + 0.5) / 8.0                                  # ties: s = 1/8 exactly
    W[5, Gs - 1] = 15.0 / 8.0
    W[5, 0] = 0.0
    W[6, g(2)] = -(k + 0.5) / 4.0                                 # ties on the negative side, z = 15
    W[6, 2 * Gs] = -15.0 / 4.0
    W[7, g(2)] = rng.standard_normal(Gs).astype(np.float32) * 3e4  # large, finite scale
    return W


@pytest.mark.parametrize("Gs", [64, 128])
@pytest.mark.parametrize("d_out,d_in", [(40, 384), (264, 1024)])
def test_quantiser_bit_exact(Gs, d_out, d_in):
    W = crafted(d_out, d_in, Gs, seed=d_out + Gs)
    q_ref, s_ref, z_ref = O.quantize_rtn(W, Gs)
    wq, sc, zp = gpu_quantize(W, Gs)
    assert np.array_equal(sc, s_ref)
    assert np.array_equal(zp, z_ref)
    assert np.array_equal(wq, O.pack_int4(q_ref))


def test_quantise_prepare_dequantise_round_trip():
    # the whole storage chain on the GPU: quantise, prepare, and the inspection hook reads
    # back exactly the oracle's dequantised weight
    Gs, act = 128, "f16"
    W = crafted(136, 512, Gs, seed=9)
    W[3] = W[8]                      # (no scale past the binary16 range here: inf * 0 has no value)
    w = torch.from_numpy(W).cuda()
    wq = torch.empty((136, 512 // 8), dtype=torch.int32, device="cuda")
    sc = torch.empty((136, 512 // Gs), dtype=torch.int16, device="cuda")
    zp = torch.empty_like(sc)
    G.glowq_quantize_rtn(w.data_ptr(), 136, 512, Gs, wq.data_ptr(), sc.data_ptr(), zp.data_ptr(), stream())
    prep = torch.empty(G.glowq_prepared_bytes(136, 512, Gs), dtype=torch.uint8, device="cuda")
    G.glowq_prepare_weights(wq.data_ptr(), sc.data_ptr(), zp.data_ptr(), 136, 512, Gs, prep.data_ptr(), stream())
    out = torch.empty((136, 512), dtype=torch.int16, device="cuda")
    G.glowq_debug_dequant(prep.data_ptr(), 136, 512, Gs, G.GLOWQ_F16, out.data_ptr(), stream())
    torch.cuda.synchronize()
    q_ref, s_ref, z_ref = O.quantize_rtn(W, Gs)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), O.dequant_bits(q_ref, s_ref, z_ref, Gs, act))
