"""GPU parity, forward (Sec. 3.3, Eqs. 8-9) at sizes the oracle finishes in
seconds: the tiny workload through both kernel paths, ragged shapes, every rank,
the restore gating, and the identities the paper fixes."""
import numpy as np
import pytest
import torch

import paper_2603_25385_amd as G
from glowq_inputs import CONFIGS, UnitShape
from oracle import glowq_oracle as O
from gpu_util import DeviceUnit, Workspace, run_group, stream
from util import recipe_unit, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-3                     # max relative error, fp32 accumulation
ULP = {"f16": 2.0 ** -11, "bf16": 2.0 ** -8}


def _check(ys, refs, tol):
    for y, ref in zip(ys, refs):
        assert y.shape == ref.shape
        assert np.isfinite(y).all()
        e = rel_err(y, ref)
        assert e <= tol, e


@pytest.mark.parametrize("T", [16, 1, 5, 32, 33, 100, 300])
def test_tiny_workload(T):
    u = recipe_unit(O, 1, 0, T)
    ys, _, _ = run_group(u, True)
    _check(ys, O.group_forward(u, True), TOL)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("T", [1, 3, 9, 20, 70, 257])
def test_ragged_group(act, T):
    # rows not a multiple of 32, three module sizes, two quantisation groups; 26 row blocks:
    # the three-block groups of the 4 < T <= 32 path straddle the modules and end ragged
    shape = UnitShape("g", 384, (40, 264, 96))
    u = recipe_unit(O, 1, 0, T, r=24, shape=shape, act=act, G=128)
    ys, _, _ = run_group(u, True, ldy_pad=8)
    _check(ys, O.group_forward(u, True), TOL)
    ys16, _, _ = run_group(u, True, out="act")
    _check(ys16, O.group_forward(u, True), TOL + ULP[act])


@pytest.mark.parametrize("r", [8, 16, 24, 32, 40, 64, 72, 120, 128])
@pytest.mark.parametrize("T", [2, 12, 32, 48])
def test_every_rank(r, T):
    shape = UnitShape("g", 256, (128, 64))
    u = recipe_unit(O, 1, 0, T, r=r, shape=shape, G=64)
    ys, _, _ = run_group(u, True)
    _check(ys, O.group_forward(u, True), TOL)


@pytest.mark.parametrize("T", [1, 3, 4, 20, 32, 70, 200])
def test_bf16_with_group_size_64(T):
    # bfloat16 activations with two quantisation groups per 128-channel tile, ragged rows
    shape = UnitShape("g", 384, (40, 264, 96))
    u = recipe_unit(O, 1, 0, T, r=24, shape=shape, act="bf16", G=64)
    ys, _, _ = run_group(u, True, ldy_pad=8)
    _check(ys, O.group_forward(u, True), TOL)
    ys16, _, _ = run_group(u, True, out="act")
    _check(ys16, O.group_forward(u, True), TOL + ULP["bf16"])
    off, _, _ = run_group(u, False, ldy_pad=16)
    _check(off, O.group_forward(u, False), TOL)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("T", [40, 130, 300])
def test_long_contraction(act, T):
    # d_in past 2048: the projection tiles of the tiled path work in K parts (here three
    # of unequal length) and the last one to finish adds them; T = 130 ends in a token
    # tile of a single 16-token block.  Twice through one workspace: the parts' arrival
    # counter must be back at zero.
    shape = UnitShape("g", 4352, (64, 40))
    u = recipe_unit(O, 1, 0, T, r=24, shape=shape, act=act, G=128)
    du = DeviceUnit(u)
    ws = Workspace([du.desc])
    ref = O.group_forward(u, True)
    for _ in range(2):
        du.clear()
        G.glowq_group_forward(du.desc, True, ws.ptr, ws.bytes, stream())
        _check(du.outputs(), ref, TOL)
        ws.assert_idle()


@pytest.mark.parametrize("act,d_in,T,out", [("f16", 8192, 70, "f32"), ("bf16", 8320, 130, "act"),
                                           ("f16", 12288, 200, "act"), ("bf16", 16384, 65, "f32")])
def test_long_contraction_in_k_slices(act, d_in, T, out):
    # 8192 channels and more on a handful of tiles: the launch cuts K into two to four slices
    # (65 tiles into 32 + 33, 96 into three, 128 into four), each slice leaves an fp32 slab in
    # the workspace, the first carries the correction, a second kernel adds them in slice
    # order; ragged rows (40: a slab row of 40 floats), padded output rows, restored and not,
    # twice through one workspace, and against a call that cannot cut (no workspace)
    shape = UnitShape("s", d_in, (40, 264))
    u = recipe_unit(O, 1, 0, T, r=24, shape=shape, act=act, G=128)
    du = DeviceUnit(u, out, 8)
    ws = Workspace([du.desc])
    tol = TOL + (ULP[act] if out == "act" else 0.0)
    seen = {}
    for restore in (True, False, True):
        du.clear()
        G.glowq_group_forward(du.desc, restore, ws.ptr, ws.bytes, stream())
        ys = du.outputs()
        _check(ys, O.group_forward(u, restore), tol)
        ws.assert_idle()
        # the slices are added in a fixed order: the same bits every time
        if restore in seen:
            assert all(np.array_equal(a, b) for a, b in zip(seen[restore], ys))
        seen[restore] = ys
    du.clear()
    G.glowq_group_forward(du.desc, False, 0, 0, stream())
    _check(du.outputs(), O.group_forward(u, False), tol)


@pytest.mark.parametrize("T", [4, 96])
def test_masked_unit_equals_rank_zero_bitwise(T):
    u = recipe_unit(O, 1, 0, T)
    off, du, ws = run_group(u, False)
    _check(off, O.group_forward(u, False), TOL)
    # rank 0 through the same buffers: identical bits
    du.clear()
    d0 = du.describe(r=0)
    G.glowq_group_forward(d0, True, ws.ptr, ws.bytes, stream())
    for a, b in zip(off, du.outputs()):
        assert np.array_equal(a, b)
    # and the restored output really differs
    on, _, _ = run_group(u, True)
    assert max(np.max(np.abs(a - b)) for a, b in zip(on, off)) > 0


@pytest.mark.parametrize("T", [7, 64])
def test_shared_projection(T):
    u = recipe_unit(O, 1, 0, T)
    du = DeviceUnit(u)
    ws = Workspace([du.desc])
    R = torch.full((T, u["r"]), float("nan"), dtype=torch.float32, device="cuda")
    G.glowq_shared_proj(du.desc, R.data_ptr(), ws.ptr, ws.bytes, stream())
    torch.cuda.synchronize()
    ref = O.shared_proj(u["X"], u["B"], u["act"])
    assert rel_err(R.double().cpu().numpy(), ref) <= 1e-5
    # a group call right after, through the same workspace, is unaffected
    G.glowq_group_forward(du.desc, True, ws.ptr, ws.bytes, stream())
    _check(du.outputs(), O.group_forward(u, True), TOL)


def test_token_independence_across_kernel_paths():
    # column t of a 48-token call (tiled GEMM path) equals the 1-token call (streaming
    # path).  The streaming path applies the group scale to the fp32 sum of x (q - z)
    # instead of multiplying with the 16-bit rounded weight, so the two paths differ by
    # the weight rounding (2^-11 per term, random sign) and by the tiled path's rounding of
    # R to 16 bits: 7e-4 of the output's rms was measured here, each path being within a
    # few 1e-4 of the oracle.
    u = recipe_unit(O, 1, 0, 48)
    many, _, _ = run_group(u, True)
    for t in (0, 17, 47):
        ut = dict(u, X=u["X"][t:t + 1], T=1)
        one, _, _ = run_group(ut, True)
        for a, b in zip(many, one):
            assert rel_err(b[0], a[t]) <= 1e-3


def test_block_forward_with_mask():
    units = [recipe_unit(O, 1, 0, T, seed=s, shape=sh, r=16, G=64)
             for s, (T, sh) in enumerate([(4, UnitShape("qkv", 256, (256, 64, 64))),
                                          (4, UnitShape("o", 256, (256,))),
                                          (40, UnitShape("gu", 128, (384, 384))),
                                          (40, UnitShape("down", 384, (128,)))])]
    mask = [1, 0, 1, 0]
    dus = [DeviceUnit(u) for u in units]
    ws = Workspace([d.desc for d in dus])
    for _ in range(2):                  # twice through the same workspace
        for d in dus:
            d.clear()
        G.glowq_block_forward([d.desc for d in dus], bytes(mask), ws.ptr, ws.bytes, stream())
        for d, u, f in zip(dus, units, mask):
            _check(d.outputs(), O.group_forward(u, bool(f)), TOL)
        ws.assert_idle()


def test_block_forward_with_k_slices_and_a_full_module_table():
    """Seven units of 70 tokens in one call, five of them with a contraction long enough to be
    cut into K slices (four slices at 16384 channels, two at 8192): the launch's table of 16
    module entries has room for some of the slices only, so units cut four ways, units cut two
    ways or not at all and ordinary units share a launch (longest contraction first, which is
    not the order of the call); masked and restored units, twice through one workspace."""
    shapes = [UnitShape("a", 256, (64, 40)), UnitShape("d1", 16384, (40,)), UnitShape("d2", 8192, (40, 24)),
              UnitShape("d3", 16384, (24,)), UnitShape("b", 384, (136,)), UnitShape("d4", 16384, (40,)),
              UnitShape("d5", 8192, (72,))]
    mask = [1, 1, 0, 1, 1, 0, 1]
    units = [recipe_unit(O, 1, 0, 70, seed=30 + i, shape=sh, r=16, G=128) for i, sh in enumerate(shapes)]
    dus = [DeviceUnit(u) for u in units]
    ws = Workspace([d.desc for d in dus])
    refs = [O.group_forward(u, bool(f)) for u, f in zip(units, mask)]
    for _ in range(2):
        for d in dus:
            d.clear()
        G.glowq_block_forward([d.desc for d in dus], bytes(mask), ws.ptr, ws.bytes, stream())
        for d, ref in zip(dus, refs):
            _check(d.outputs(), ref, TOL)
        ws.assert_idle()


def test_block_forward_mixed_token_counts():
    """Thirteen few-token units of different token classes and gating in one call: the
    decode launches batch up to eight compatible units and must split at every change
    of class; every unit's result is the single-unit result."""
    Ts = [1, 1, 2, 1, 1, 1, 1, 1, 1, 1, 4, 9, 1]
    mask = [1, 0, 1, 1, 1, 0, 1, 1, 1, 1, 1, 1, 0]
    shapes = [UnitShape("a", 256, (64, 32)), UnitShape("b", 128, (48,)), UnitShape("c", 384, (16, 16, 16))]
    units = [recipe_unit(O, 1, 0, T, seed=10 + i, shape=shapes[i % 3], r=16, G=64)
             for i, T in enumerate(Ts)]
    dus = [DeviceUnit(u) for u in units]
    ws = Workspace([d.desc for d in dus])
    for _ in range(2):
        for d in dus:
            d.clear()
        G.glowq_block_forward([d.desc for d in dus], bytes(mask), ws.ptr, ws.bytes, stream())
        for d, u, f in zip(dus, units, mask):
            _check(d.outputs(), O.group_forward(u, bool(f)), TOL)
        ws.assert_idle()


@pytest.mark.parametrize("T", [1, 12, 40])
def test_graph_replay_matches_eager(T):
    """A captured group forward replayed several times, with new activations written
    into the same buffers between replays, gives the eager result every time (the
    single-launch decode path must tell one replay's projection from the previous)."""
    u = recipe_unit(O, 1, 0, T)
    du = DeviceUnit(u)
    ws = Workspace([du.desc])
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        G.glowq_group_forward(du.desc, True, ws.ptr, ws.bytes, side.cuda_stream)   # warm-up
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            G.glowq_group_forward(du.desc, True, ws.ptr, ws.bytes,
                                  torch.cuda.current_stream().cuda_stream)
    from glowq_inputs import gen_activations
    from gpu_util import dev_bits
    for rep in range(4):
        xb = gen_activations(100 + rep, 0, T, u["d_in"], u["act"], False)
        du.X.copy_(dev_bits(xb))
        du.clear()
        torch.cuda.synchronize()
        graph.replay()
        got = du.outputs()
        ref = O.group_forward(dict(u, X=xb), True)
        _check(got, ref, TOL)
        # eager work and a synchronisation between the replays
        du.clear()
        G.glowq_group_forward(du.desc, True, ws.ptr, ws.bytes, stream())
        _check(du.outputs(), ref, TOL)
    ws.assert_idle()
