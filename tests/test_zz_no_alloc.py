"""GPU check of glowq_group_forward_static, the entry point that allocates nothing: its
output equals glowq_group_forward's on two calls in a row through the one scratch array,
the second with a smaller input laid out differently (tiled path, then streaming path),
and a unit whose scratch need exceeds the array is refused."""
import numpy as np
import pytest
import torch

import paper_2603_25385_amd as G
from glowq_inputs import UnitShape
from oracle import glowq_oracle as O
from gpu_util import DeviceUnit, Workspace, stream
from util import recipe_unit, rel_err

pytestmark = pytest.mark.gpu


def _both(u, restore):
    du = DeviceUnit(u)
    ws = Workspace([du.desc])
    G.glowq_group_forward(du.desc, restore, ws.ptr, ws.bytes, stream())
    ref = du.outputs()
    du.clear()
    G.glowq_group_forward_static(du.desc, restore, stream())
    got = du.outputs()
    return ref, got


def test_static_scratch_entry_point_matches_the_workspace_one():
    big = recipe_unit(O, 1, 0, 300, r=24, shape=UnitShape("g", 4352, (64, 40)), G=128)   # K parts
    small = recipe_unit(O, 1, 0, 3, r=16, shape=UnitShape("s", 256, (96, 32)), G=64)
    for u in (big, small, big):
        for restore in (True, False):
            ref, got = _both(u, restore)
            oracle = O.group_forward(u, restore)
            for a, b, o in zip(ref, got, oracle):
                assert np.isfinite(b).all()
                assert np.array_equal(a, b)
                assert rel_err(b, o) <= 2e-3


def test_static_scratch_refuses_what_does_not_fit():
    # T x r x parts of fp32 partial sums well past 16 MiB; checked on the host, nothing runs
    mods = [G.make_module(0x3000, 0x4000, 0x5000, 64, 64)]
    u = G.make_unit(0x1000, 0x2000, mods, 1 << 17, 4096, 128, 128, G.GLOWQ_F16, G.GLOWQ_F32)
    assert G.glowq_workspace_bytes([u]) > G.GLOWQ_STATIC_SCRATCH_BYTES
    with pytest.raises(G.GlowqError) as e:
        G.glowq_group_forward_static(u, True, 0)
    assert e.value.status == G.GLOWQ_ERR_WORKSPACE
