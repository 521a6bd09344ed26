"""GPU parity of the importance scores of GlowQ-S (Sec. 3.3, Eqs. 10-11) and of the
selection they feed: the library's float64 reductions over the full-precision weights, the
prepared layout and the stored factors against the oracle's definitions."""
import numpy as np
import pytest
import torch

import paper_2603_25385_amd as G
from glowq_inputs import UnitShape
from oracle import glowq_oracle as O
from gpu_util import DeviceUnit, stream
from util import recipe_unit

pytestmark = pytest.mark.gpu
REL = 1e-10        # float64 sums of up to 10^5 terms, added in a different order


def _gpu_scores(u):
    du = DeviceUnit(u)
    Ws = [torch.from_numpy(np.ascontiguousarray(w, np.float32)).cuda() for w in u["W"]]
    scratch = torch.full((G.GLOWQ_IMPORTANCE_SCRATCH_BYTES // 8,), float("nan"), dtype=torch.float64, device="cuda")
    scores = torch.full((4,), float("nan"), dtype=torch.float64, device="cuda")
    G.glowq_unit_importance(du.desc, [w.data_ptr() for w in Ws], scratch.data_ptr(), scores.data_ptr(), stream())
    torch.cuda.synchronize()
    out = scores.cpu().numpy()
    assert np.isnan(out[2:]).all()                   # only two values are written
    return float(out[0]), float(out[1])


def _oracle_scores(u):
    act, Gs = u["act"], u["G"]
    What = [O.dequant(O.unpack_int4(m["wq"]), m["scales"], m["zeros"], Gs, act) for m in u["modules"]]
    ner = O.importance_ner(u["W"], What)
    E = O.stack_errors(u["W"], What)
    energy = float(np.sum(E ** 2))
    if u["r"] == 0:
        return ner, 0.0, 0.0
    stored = O.importance_ec_from_factors([m["A"] for m in u["modules"]], u["B"], act, energy)
    return ner, stored, O.importance_ec(E, u["r"])


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("Gs", [64, 128])
def test_scores_match_the_oracle(act, Gs):
    shape = UnitShape("g", 384, (40, 264, 96))       # ragged row blocks, three modules
    u = recipe_unit(O, 1, 0, 4, r=24, shape=shape, act=act, G=Gs)
    ner, ec = _gpu_scores(u)
    ner_ref, ec_stored, ec_spectrum = _oracle_scores(u)
    assert ner == pytest.approx(ner_ref, rel=REL)
    assert ec == pytest.approx(ec_stored, rel=REL)
    assert ec == pytest.approx(ec_spectrum, rel=2e-2 if act == "bf16" else 3e-3)   # 16-bit factors
    assert 0.0 < ec < 1.0 and 0.0 < ner < 0.1


def test_rank_zero_and_full_size_unit():
    u0 = recipe_unit(O, 1, 0, 4, r=0, shape=UnitShape("g", 256, (64, 64)), G=64)
    ner, ec = _gpu_scores(u0)
    assert ec == 0.0 and ner == pytest.approx(_oracle_scores(u0)[0], rel=REL)
    u = recipe_unit(O, 1, 0, 4)                      # the tiny workload's q/k/v group
    ner, ec = _gpu_scores(u)
    ref = _oracle_scores(u)
    assert ner == pytest.approx(ref[0], rel=REL) and ec == pytest.approx(ref[1], rel=REL)


def test_scores_rank_units_like_the_oracle():
    # four units of different shapes and ranks; the selection from the GPU's scores is the
    # oracle's for every k
    shapes = [UnitShape("a", 256, (64, 128)), UnitShape("b", 384, (40,)), UnitShape("c", 256, (136, 16, 64)),
              UnitShape("d", 128, (96, 32))]
    units = [recipe_unit(O, 1, i, 4, r=8 * (i + 1), shape=s, G=128, seed=40 + i) for i, s in enumerate(shapes)]
    gpu = [_gpu_scores(u) for u in units]
    ref = [_oracle_scores(u) for u in units]
    for which in (0, 1):
        a = [g[which] for g in gpu]
        b = [r[which] for r in ref]
        for k in range(len(units) + 1):
            assert G.glowq_select_units(a, k) == O.select_units(b, k).tolist()
