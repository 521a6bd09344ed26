"""GPU parity of the layer-wise comparison mode (the latency study's "Layerwise" rows,
Sec. 4.3): every module projects with a right factor of its own.  Factors come from the
oracle's layer-wise setup (per-block truncated SVD); the expected outputs from the
oracle's layerwise_forward."""
import numpy as np
import pytest
import torch

import paper_2603_25385_amd as G
from glowq_inputs import CONFIGS, UnitShape, gen_activations, gen_module_weight
from oracle import glowq_oracle as O
from gpu_util import DeviceUnit, dev_bits, stream
from util import rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-3                     # max relative error, fp32 accumulation


def _layerwise_unit(shape, T, r, Gs, act, seed=77):
    W = [gen_module_weight(seed, 0, i, o, shape.d_in) for i, o in enumerate(shape.d_outs)]
    X = gen_activations(seed, 0, T, shape.d_in, act, True)
    return O.build_unit_layerwise(W, X, r, Gs, act)


def _run(units, ldy_pad=0):
    """All units in one call; returns their outputs."""
    dus = [DeviceUnit(dict(u, B=u["modules"][0]["B"]), "f32", ldy_pad) for u in units]  # (own B ignored)
    Bs = [dev_bits(m["B"]) for u in units for m in u["modules"]]
    assert all(tuple(b.shape) == (du.r, du.d_in) for b, du in zip(Bs, [d for d in dus for _ in d.modules]))
    descs = [du.desc for du in dus]
    nbytes = G.glowq_layerwise_workspace_bytes(descs)
    # one slice per module, each as long as that one-module unit's workspace
    solo, j = [], 0
    for du in dus:
        for i in range(len(du.modules)):
            one = G.make_unit(du.X.data_ptr(), Bs[j].data_ptr(), [du.desc.modules[i]], du.T, du.d_in,
                              du.r, du.Gs, du.desc.act_dtype, du.desc.out_dtype)
            solo.append(G.glowq_workspace_bytes([one]))
            j += 1
    assert nbytes == sum(solo)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    G.glowq_workspace_init(ws.data_ptr(), nbytes, stream())
    G.glowq_layerwise_forward(descs, [b.data_ptr() for b in Bs], ws.data_ptr(), nbytes, stream())
    ys = [du.outputs() for du in dus]
    # no slice reports a dropped correction (word 3 of each module's slice)
    words = ws.view(torch.int32).cpu().numpy()
    off = 0
    for n in solo:
        assert words[off // 4 + 3] == 0
        off += n
    return ys


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("T", [1, 2, 4, 9, 32, 70, 257])
def test_layerwise_matches_the_oracle(act, T):
    shape = UnitShape("g", 384, (40, 264, 96))
    u = _layerwise_unit(shape, T, 24, 128, act)
    refs = O.layerwise_forward(u)
    for y, ref in zip(_run([u], ldy_pad=8)[0], refs):
        assert y.shape == ref.shape and np.isfinite(y).all()
        assert rel_err(y, ref) <= TOL
    # the factors differ per module, so the shared forward with any one of them must not
    # reproduce the layer-wise outputs of the others
    wrong = O.group_forward(dict(u, B=u["modules"][0]["B"]), True)
    assert rel_err(wrong[1], refs[1]) > 10 * TOL


@pytest.mark.parametrize("T", [1, 16, 130])
def test_layerwise_block_of_units(T):
    # several units of different shapes in one call: the factor list runs unit after unit
    shapes = [UnitShape("a", 256, (64, 128)), UnitShape("b", 384, (40,)), UnitShape("c", 256, (136, 16, 64))]
    units = [_layerwise_unit(s, T, 16, 128, "f16", seed=90 + i) for i, s in enumerate(shapes)]
    for u, ys in zip(units, _run(units)):
        for y, ref in zip(ys, O.layerwise_forward(u)):
            assert np.isfinite(y).all() and rel_err(y, ref) <= TOL


def test_layerwise_rejects_missing_factors():
    shape = UnitShape("g", 256, (64, 64))
    u = _layerwise_unit(shape, 4, 8, 128, "f16")
    du = DeviceUnit(dict(u, B=u["modules"][0]["B"]))
    nbytes = G.glowq_layerwise_workspace_bytes([du.desc])
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    b0 = dev_bits(u["modules"][0]["B"])
    with pytest.raises(G.GlowqError) as e:
        G.glowq_layerwise_forward([du.desc], [b0.data_ptr(), 0], ws.data_ptr(), nbytes, stream())
    assert e.value.status == G.GLOWQ_ERR_NULL
    with pytest.raises(G.GlowqError) as e:
        G.glowq_layerwise_forward([du.desc], [b0.data_ptr(), b0.data_ptr()], ws.data_ptr(), nbytes - 16, stream())
    assert e.value.status == G.GLOWQ_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert all(torch.isnan(y).all() for y in du.Y)      # nothing was enqueued
